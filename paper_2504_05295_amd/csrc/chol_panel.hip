// The r x r Cholesky factorisation of Cholesky-QR (Appendix A), blocked right-looking with 64-wide panels.
// Two drivers share the code for the 64 x 64 diagonal block: one launch per panel with no dependency between
// workgroups (below; large batches), and the whole factorisation in one launch with workgroups that hand
// results on through flags (chol_stream_kernel further down; one to four matrices).
//
// One panel step as a single launch:
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
//   wave 0  eliminates C11 column by column on unscaled values (row i of the block lives in the registers
//           of lane i); it carries the chain of dependent pivots and does nothing that is not on it,
//   wave 2  follows and scales the raw columns into columns of L11 (reciprocal square roots, bounds check),
//   wave 1  follows wave 0 as well and builds W11 = L11^-1 by forward substitution on the raw columns,
//   wave 3  meanwhile fetches the two panel blocks C21_i, C21_j into LDS.
// The waves talk through LDS: broadcast reads (all lanes read one address) replace cross-lane shuffles, and
// counters tell the followers which columns are final.  LDS operations of one wave are processed in issue
// order, so data stored before a counter is visible to whoever sees the counter.
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

// LDS pointers carry their address space, so that volatile accesses too become ds_* instructions (a volatile
// access through a generic pointer is a flat one, with a much longer round trip).
typedef __attribute__((address_space(3))) float lds_float;
typedef __attribute__((address_space(3))) f32x4_t lds_f32x4;
typedef __attribute__((address_space(3))) volatile int lds_counter;

__device__ __forceinline__ float lane_value(float x, int src_lane) {   // x of lane `src_lane`, uniform result
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), src_lane));
}

// Wave 0: eliminates the 64x64 block held in S0 (row i in lane i), right-looking, one column per step,
// working on raw (unscaled) values: with g = a[i][j] / a[j][j] the update is a[i][k] -= g * a[k][j], which
// equals L[i][j] L[k][j].  The dependency chain from one pivot to the next is kept free of LDS round trips:
// the pivot and the two entries of the column that the next two columns need come through lane reads, and
// column j's update of the entries further right (k >= j+3) is applied one step late, from the copy of the
// raw column that went through LDS meanwhile.  Raw column j is left in row j of S0 (its first reader, this
// wave, took the whole block into registers before the first column is written) and *raw_done counts them.
// RANK (the factorisation that tolerates linearly dependent columns): a column whose pivot is not above its
// threshold thr[j] (a fraction of the Gram matrix' original diagonal entry) is dependent on the columns before it; it
// eliminates nothing, so that the factorisation goes on as if the column were not there.  The two follower waves
// take the same decision from the same two numbers.
template <bool RANK>
__device__ __forceinline__ void eliminate_wave(lds_float* S0, lds_counter* raw_done, int lane, const float* thr) {
    float a[CB];
    float thr_lane = 0.f;
    if constexpr (RANK) thr_lane = thr[lane];
    static_for<0, CB>([&](auto kc) __attribute__((always_inline)) { a[decltype(kc)::value] = S0[lane * CBP + decltype(kc)::value]; });
    f32x4_t cv0[CB / 4], cv1[CB / 4];   // raw columns j (even / odd) as read back from LDS
    float gprev = 0.f;
    static_for<0, CB>([&](auto jc) __attribute__((always_inline)) {
      constexpr int jj = decltype(jc)::value;
      f32x4_t* cur = (jj & 1) ? cv1 : cv0;
      const f32x4_t* prev = (jj & 1) ? cv0 : cv1;
      const float piv = lane_value(a[jj], jj);
      float gj = a[jj] * __builtin_amdgcn_rcpf(piv);
      if constexpr (RANK) {
        if (!(piv > lane_value(thr_lane, jj))) gj = 0.f;   // uniform
      }
      if constexpr (jj + 1 < CB) a[jj + 1] -= gj * lane_value(a[jj], jj + 1);
      if constexpr (jj + 2 < CB) {
        if constexpr (jj >= 1) a[jj + 2] -= gprev * prev[(jj + 2) / 4][(jj + 2) % 4];
        a[jj + 2] -= gj * lane_value(a[jj], jj + 2);
      }
      lds_float* cb = S0 + jj * CBP;
      cb[lane] = a[jj];
      if constexpr (jj + 3 < CB) {
        // entries below j+3 of the first group of four are not read at all: their registers would be reused at
        // once, and the hardware then waits for the read before it lets them be overwritten
        constexpr int q0 = (jj + 3) / 4;
        static_for<jj + 3, (4 * q0 + 4 < CB ? 4 * q0 + 4 : CB)>([&](auto kc) __attribute__((always_inline)) {
          constexpr int k = decltype(kc)::value;
          cur[q0][k % 4] = cb[k];
        });
        static_for<q0 + 1, CB / 4>([&](auto qc) __attribute__((always_inline)) {
          constexpr int q = decltype(qc)::value;
          cur[q] = *(const lds_f32x4*)(cb + 4 * q);
        });
      }
      asm volatile("" ::: "memory");
      *raw_done = jj + 1;
      // the reads above stay in flight across the rest of this step; nothing below may move up past them
      __builtin_amdgcn_sched_barrier(0);
      // late part of column j-1's update
      if constexpr (jj >= 1) {
        static_for<(jj + 3) / 4, CB / 4>([&](auto qc) __attribute__((always_inline)) {
          constexpr int q = decltype(qc)::value;
          if constexpr (4 * q + 0 >= jj + 3) a[4 * q + 0] -= gprev * prev[q][0];
          if constexpr (4 * q + 1 >= jj + 3) a[4 * q + 1] -= gprev * prev[q][1];
          if constexpr (4 * q + 2 >= jj + 3) a[4 * q + 2] -= gprev * prev[q][2];
          if constexpr (4 * q + 3 >= jj + 3) a[4 * q + 3] -= gprev * prev[q][3];
        });
      }
      gprev = gj;
      __builtin_amdgcn_sched_barrier(0);
    });
}

// Wave 2: follows wave 0 and turns raw columns into columns of L: L[i][j] = raw[i][j] / sqrt(raw[j][j]).
// Leaves 1 / sqrt(raw[j][j]) in rsv and sets *scaled when all of them are there.  When Lout is given
// (writer workgroup) also stores L11 and the status.
// RANK: a dependent column (pivot not above thr[j]) becomes a zero column of L with a zero diagonal entry and 0 in rsv,
// which makes row and column j of the inverse zero as well; nullmask[j] (writer only) records the decision.
template <bool RANK>
__device__ __forceinline__ void scale_wave(const lds_float* S0, lds_counter* raw_done, lds_float* rsv, lds_counter* scaled, int lane,
                                           float piv_lo, float piv_hi, float* Lout, long long ld, int* status, const float* thr,
                                           int* nullmask) {
    float l[CB];
    bool bad = false;
    int seen = 0;
    float raw0 = 0.f, raw1 = 0.f, piv0 = 1.f, piv1 = 1.f;
    // column j+1 is fetched while column j is being scaled; a column is only asked for once it is final
    auto fetch = [&](auto jc, float& raw, float& piv) __attribute__((always_inline)) {
      constexpr int jj = decltype(jc)::value;
      if (seen <= jj) {
        do { seen = *raw_done; } while (seen <= jj);   // wave 0 always gets there: it waits for nobody
      }
      asm volatile("" ::: "memory");
      raw = S0[jj * CBP + lane];
      piv = S0[jj * CBP + jj];
    };
    fetch(std::integral_constant<int, 0>{}, raw0, piv0);
    static_for<0, CB>([&](auto jc) __attribute__((always_inline)) {
      constexpr int jj = decltype(jc)::value;
      const float raw = (jj & 1) ? raw1 : raw0, piv = (jj & 1) ? piv1 : piv0;
      if constexpr (jj + 1 < CB) fetch(std::integral_constant<int, jj + 1>{}, (jj & 1) ? raw0 : raw1, (jj & 1) ? piv0 : piv1);
      __builtin_amdgcn_sched_barrier(0);
      float rs = __builtin_amdgcn_rsqf(piv);
      rs = rs * (1.5f - 0.5f * piv * rs * rs);   // one Newton step on the hardware estimate
      if constexpr (RANK) {
        const bool dependent = !(piv > thr[jj]);
        if (dependent) rs = 0.f;
        bad = bad || !(piv == piv) || (!dependent && (!(piv > piv_lo) || !(piv < piv_hi)));   // a NaN pivot is no dependent column
        if (nullmask && lane == 0) nullmask[jj] = dependent ? 1 : 0;
      } else {
        bad = bad || !(piv > piv_lo) || !(piv < piv_hi);
      }
      l[jj] = raw * rs;
      rsv[jj] = rs;   // every lane stores the same value
      asm volatile("" : "+v"(l[jj]));   // keeps this column's arithmetic from being moved past the next wait loop
      __builtin_amdgcn_sched_barrier(0);
    });
    asm volatile("" ::: "memory");
    *scaled = 1;
    if (Lout) {
      static_for<0, CB>([&](auto kc) __attribute__((always_inline)) {
        constexpr int k = decltype(kc)::value;
        Lout[(long long)lane * ld + k] = (k <= lane) ? l[k] : 0.f;
      });
      if (bad && lane == 0 && *status == 0) *status = ST_BREAKDOWN;   // a code that is already there (an earlier stage failed) stays
    }
}

// Wave 1: W11 = L11^-1, following wave 0 column by column; leaves W11 (row-major) in S0.
// Lane c builds column c of W by forward substitution in its right-looking form, on raw values as well:
// with acc_i = delta_ic - sum_{k<j} L[i][k] w_k, step j sets acc_i -= raw[i][j] * (acc_j / raw[j][j]) for i > j,
// and w_j = acc_j / sqrt(raw[j][j]) is applied to all rows at the end.  The work per step shrinks as the
// elimination's does, so this wave finishes right behind wave 0.
template <bool RANK>
__device__ __forceinline__ void invert_wave(lds_float* S0, lds_counter* raw_done, const lds_float* rsv, lds_counter* scaled, int lane,
                                            const float* thr) {
    float w[CB];
    static_for<0, CB>([&](auto ic) __attribute__((always_inline)) { w[decltype(ic)::value] = (lane == decltype(ic)::value) ? 1.f : 0.f; });
    f32x4_t cv0[CB / 4], cv1[CB / 4];
    float piv0 = 1.f, piv1 = 1.f;
    int seen = 0;
    // raw column j+1 is fetched while column j is being used; a column is only asked for once it is final
    auto fetch = [&](auto jc, f32x4_t* cv, float& piv) __attribute__((always_inline)) {
      constexpr int jj = decltype(jc)::value;
      if (seen <= jj) {
        do { seen = *raw_done; } while (seen <= jj);   // wave 0 always gets there: it waits for nobody
      }
      asm volatile("" ::: "memory");
      const lds_float* cb = S0 + jj * CBP;
      piv = cb[jj];
      if constexpr (jj + 1 < CB) {
        constexpr int q0 = (jj + 1) / 4;   // entries up to j of the first group of four are not read (see wave 0)
        static_for<jj + 1, (4 * q0 + 4 < CB ? 4 * q0 + 4 : CB)>([&](auto kc) __attribute__((always_inline)) {
          constexpr int k = decltype(kc)::value;
          cv[q0][k % 4] = cb[k];
        });
        static_for<q0 + 1, CB / 4>([&](auto qc) __attribute__((always_inline)) {
          constexpr int q = decltype(qc)::value;
          cv[q] = *(const lds_f32x4*)(cb + 4 * q);
        });
      }
    };
    fetch(std::integral_constant<int, 0>{}, cv0, piv0);
    static_for<0, CB>([&](auto jc) __attribute__((always_inline)) {
      constexpr int jj = decltype(jc)::value;
      const f32x4_t* cv = (jj & 1) ? cv1 : cv0;
      const float piv = (jj & 1) ? piv1 : piv0;
      if constexpr (jj + 1 < CB) fetch(std::integral_constant<int, jj + 1>{}, (jj & 1) ? cv0 : cv1, (jj & 1) ? piv0 : piv1);
      __builtin_amdgcn_sched_barrier(0);
      float u = w[jj] * __builtin_amdgcn_rcpf(piv);
      if constexpr (RANK) {
        if (!(piv > thr[jj])) u = 0.f;   // a dependent column takes no part in the substitution
      }
      static_for<(jj + 1) / 4, CB / 4>([&](auto qc) __attribute__((always_inline)) {
        constexpr int q = decltype(qc)::value;
        if constexpr (4 * q + 0 > jj) w[4 * q + 0] -= cv[q][0] * u;
        if constexpr (4 * q + 1 > jj) w[4 * q + 1] -= cv[q][1] * u;
        if constexpr (4 * q + 2 > jj) w[4 * q + 2] -= cv[q][2] * u;
        if constexpr (4 * q + 3 > jj) w[4 * q + 3] -= cv[q][3] * u;
      });
      // keeps this step's arithmetic from being moved past the next wait loop
      static_for<jj + 1, CB>([&](auto kc) __attribute__((always_inline)) {
        float& wk = w[decltype(kc)::value];
        asm volatile("" : "+v"(wk));
      });
      __builtin_amdgcn_sched_barrier(0);
    });
    while (*scaled == 0) __builtin_amdgcn_s_sleep(1);   // wave 2 always gets there: it waits only for wave 0
    asm volatile("" ::: "memory");
    // waves 0 and 2 are through with S0 by now
    static_for<0, CB>([&](auto rc) __attribute__((always_inline)) {
      constexpr int rr = decltype(rc)::value;
      S0[rr * CBP + lane] = w[rr] * rsv[rr];
    });
}

template <bool RANK>
__global__ void __launch_bounds__(256, 2) chol_panel_kernel(CholPanelPtrs p, int k0, int rp, float piv_lo, float piv_hi, int mode) {
  // mode 0: fused (workgroup 0 writes L11/W11, the others own tiles and redo the factorisation)
  // mode 1: diagonal block only (one workgroup per matrix)      mode 2: tiles only, W11 read back from memory
  // Modes 1+2 are used when there are so many tiles (large batches) that redoing the factorisation in
  // every workgroup would cost more than a second launch.
  const long long mat = (long long)blockIdx.y * p.stride;
  float* C = p.C + mat;
  float* L = p.L + mat;
  float* W = p.W + mat;
  int* status = p.status + blockIdx.y;
  const float* thr = RANK ? p.thr + mat + k0 : nullptr;
  int* nullmask = RANK ? p.nullmask + mat + k0 : nullptr;
  // Only the second Cholesky-QR pass carries a skip flag (set when it needs no factorisation); the first pass
  // starts its loads without this extra memory round trip.
  if (p.skip && p.skip[mat] != 0) return;   // uniform for the whole workgroup
  const long long ld = rp;
  __shared__ __attribute__((aligned(16))) float S0[CB * CBP];   // C11, later W11
  __shared__ __attribute__((aligned(16))) float S1[CB * CBP];   // C21_i, later L21_i
  __shared__ __attribute__((aligned(16))) float S2[CB * CBP];   // C21_j, later L21_j
  __shared__ float rsv[CB];                                     // 1 / L[j][j]
  __shared__ volatile int scaled;                               // set when rsv is complete
  __shared__ volatile int raw_done;                             // number of eliminated (raw) columns
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

  for (int idx = t; idx < CB * CB / 4; idx += 256) {
    const int rr = idx >> 4, cc = (idx & 15) * 4;
    const long long at = (long long)(k0 + rr) * ld + k0 + cc;
    f32x4_t v = *(const f32x4_t*)((mode == 2) ? W + at : C + at);
    if (mode != 2) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (cc + e > rr) v[e] = 0.f;
    }
    *(f32x4_t*)(S0 + rr * CBP + cc) = v;
  }
  if (t == 0) { scaled = 0; raw_done = 0; }
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
    for (int idx = t; idx < CB * CB / 4; idx += 256) {
      const int rr = idx >> 4, cc = (idx & 15) * 4;
      *(f32x4_t*)(S1 + rr * CBP + cc) = *(const f32x4_t*)(C + (rowi + rr) * ld + k0 + cc);
      if (j != i) *(f32x4_t*)(S2 + rr * CBP + cc) = *(const f32x4_t*)(C + (rowj + rr) * ld + k0 + cc);
    }
  } else if (wave == 0) {
    eliminate_wave<RANK>((lds_float*)S0, (lds_counter*)&raw_done, lane, thr);
  } else if (wave == 2) {
    scale_wave<RANK>((const lds_float*)S0, (lds_counter*)&raw_done, (lds_float*)rsv, (lds_counter*)&scaled, lane, piv_lo, piv_hi,
                     writer ? L + (long long)k0 * ld + k0 : nullptr, ld, status, thr, writer ? nullmask : nullptr);
  } else if (wave == 1) {
    invert_wave<RANK>((lds_float*)S0, (lds_counter*)&raw_done, (const lds_float*)rsv, (lds_counter*)&scaled, lane, thr);
  } else if (!writer) {
    for (int idx = lane; idx < CB * CB / 4; idx += 64) {
      const int rr = idx >> 4, cc = (idx & 15) * 4;
      *(f32x4_t*)(S1 + rr * CBP + cc) = *(const f32x4_t*)(C + (rowi + rr) * ld + k0 + cc);
      if (j != i) *(f32x4_t*)(S2 + rr * CBP + cc) = *(const f32x4_t*)(C + (rowj + rr) * ld + k0 + cc);
    }
  }
  __syncthreads();
  if (writer) {
    for (int idx = t; idx < CB * CB / 4; idx += 256) {
      const int rr = idx >> 4, cc = (idx & 15) * 4;
      *(f32x4_t*)(W + (long long)(k0 + rr) * ld + k0 + cc) = *(const f32x4_t*)(S0 + rr * CBP + cc);
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

// ---------------------------------------------------------------------------------------------------------
// The whole factorisation in one launch, for one or a few matrices (where a launch per panel leaves the GPU
// waiting on launch latencies and on workgroups that each redo the diagonal block).
//
// The 64x64 tiles of the lower triangle have fixed owners: tile (i, j) belongs to workgroup
// (i mod pr) * pc + (j mod pc), except that (i, i-1) goes with (i, i).  An owner does everything that
// happens to its tile, in panel order k = 0, 1, ...:
//   D(k)      tile (k, k):        factor it, publish L11, W11 = L11^-1                  -> wflag[k]
//   T(i, k)   tile (i, k), i > k: L[i][k] = C[i][k] W11^T, publish it                   -> lflag[i] = k + 1
//   U(i,j,k)  tile (i, j), j > k: C[i][j] -= L[i][k] L[j][k]^T                          (needs lflag[i], lflag[j] > k)
// so tile data never changes hands; only W11 and the finished tiles of L cross between workgroups, through
// memory, with device-scope stores and loads, each announced by a flag that is written once the stores have
// completed.  The owner of (k+1, k+1) also owns (k+1, k): the chain D(k) -> T(k+1, k) -> U(k+1, k+1, k)
// -> D(k+1), which bounds the run time, crosses workgroups once per panel, and that workgroup takes it before
// its other work.  Every workgroup handles its tasks in an order in which a task only waits for tasks that
// come earlier in the common order (panel, then D < T < U), so somebody can always proceed.
// Flags carry the number of the launch (epoch, a counter kept in device memory) and need no clearing.  Waits are bounded: a workgroup that
// gives up raises the abort word, everybody else sees it at the next wait, and the status word reports a wait
// timeout for the matrix (not a breakdown: nothing is known about its numerics); all workgroups must be resident at once, which the host guarantees by the grid size.
namespace {
typedef unsigned long long u64;
typedef __attribute__((address_space(1))) float gfloat;
typedef __attribute__((address_space(1))) int gint;
typedef __attribute__((address_space(1))) u64 gu64;
typedef __attribute__((address_space(1))) f32x4_t gf32x4;

__device__ __forceinline__ u64 flag_load(const gu64* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void flag_store(gu64* p, u64 v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Data that crosses between workgroups (W11 and the tiles of L) is written and read with device-scope
// accesses, which go past the caches that are private to a compute unit or to one part of the chip; no
// cache-wide write-back or invalidation is needed then, only that the writer's stores have completed
// before its flag goes out.
__device__ __forceinline__ float shared_load(const gfloat* p) {
  return __int_as_float(__hip_atomic_load((const gint*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void shared_store(gfloat* p, float v) {
  __hip_atomic_store((gint*)p, __float_as_int(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// 64x64 fp32 tile, global (leading dimension ld) <-> LDS (row stride CBP), by the whole workgroup.
// Thread t handles column t % 64 of rows t / 64 + 4 e.
__device__ __forceinline__ void shared_tile_to_lds(float* S, const gfloat* src, int ld, int t) {
  float v[16];
  const int r0 = t >> 6, c = t & 63;
#pragma unroll
  for (int e = 0; e < 16; ++e) v[e] = shared_load(src + (r0 + 4 * e) * ld + c);
#pragma unroll
  for (int e = 0; e < 16; ++e) S[(r0 + 4 * e) * CBP + c] = v[e];
}
// The two halves of it, so that a caller can have the loads of several tiles in flight before it waits for the first:
__device__ __forceinline__ void shared_tile_to_regs(float (&v)[16], const gfloat* src, int ld, int t) {
  const int r0 = t >> 6, c = t & 63;
#pragma unroll
  for (int e = 0; e < 16; ++e) v[e] = shared_load(src + (r0 + 4 * e) * ld + c);
}
template <bool TRANSPOSED>
__device__ __forceinline__ void regs_to_lds(float* S, const float (&v)[16], int t) {
  const int r0 = t >> 6, c = t & 63;
#pragma unroll
  for (int e = 0; e < 16; ++e) S[TRANSPOSED ? c * CBP + r0 + 4 * e : (r0 + 4 * e) * CBP + c] = v[e];
}
__device__ __forceinline__ void lds_to_shared_tile(gfloat* dst, int ld, const float* S, int t) {
  const int r0 = t >> 6, c = t & 63;
#pragma unroll
  for (int e = 0; e < 16; ++e) shared_store(dst + (r0 + 4 * e) * ld + c, S[(r0 + 4 * e) * CBP + c]);
}
__device__ __forceinline__ void tile_to_lds(float* S, const gfloat* src, int ld, int t) {
#pragma unroll
  for (int idx = t; idx < CB * CB / 4; idx += 256) {
    const int rr = idx >> 4, cc = (idx & 15) * 4;
    *(f32x4_t*)(S + rr * CBP + cc) = *(const gf32x4*)(src + rr * ld + cc);
  }
}

struct StreamCtx {
  gfloat* C;
  gfloat* L;
  gfloat* W;
  int* status;
  gu64* wflag;
  gu64* lflag;
  gu64* abort_word;
  u64 epoch;
  unsigned spin_limit;
  int ld;
  float piv_lo, piv_hi;
};

// Polls until ready() holds, on behalf of the threads with `mine`; returns false for everybody when a wait
// was given up (here or, as the abort word tells, elsewhere).
template <class F>
__device__ __forceinline__ bool wait_until(const StreamCtx& x, int* gave_up, bool mine, F ready) {
  if (mine) {
    unsigned n = 0;
    while (!ready()) {
      __builtin_amdgcn_s_sleep(2);
      if (++n > x.spin_limit) {
        flag_store(x.abort_word, x.epoch);
        if (*x.status == 0) *x.status = ST_TIMEOUT;
        *(volatile int*)gave_up = 1;
        break;
      }
      if ((n & 31u) == 0 && flag_load(x.abort_word) == x.epoch) {
        *(volatile int*)gave_up = 1;
        break;
      }
    }
  }
  __syncthreads();
  return *(volatile int*)gave_up == 0;
}
}  // namespace

template <bool RANK>
__global__ void __launch_bounds__(256, 1) chol_stream_kernel(CholStreamArgs p) {
  const long long mat = (long long)blockIdx.y * p.stride;
  if (p.skip && p.skip[mat] != 0) return;   // uniform for the whole grid row of this matrix
  const int nb = p.rp / CB, pr = p.pr, pc = p.pc;
  StreamCtx x;
  x.C = (gfloat*)(p.C + mat);
  x.L = (gfloat*)(p.L + mat);
  x.W = (gfloat*)(p.W + mat);
  x.status = p.status + blockIdx.y;
  x.wflag = (gu64*)(p.sync + (long long)blockIdx.y * p.sync_stride);
  x.lflag = x.wflag + nb;
  x.abort_word = x.lflag + nb;
  x.epoch = *p.step_counter * 8ull + (u64)p.pass;   // unique per launch: step counter kept on the device, pass within the step
  x.spin_limit = p.spin_limit;
  x.ld = p.rp;
  x.piv_lo = p.piv_lo;
  x.piv_hi = p.piv_hi;
  const int ld = p.rp;
  const float* thr = RANK ? p.thr + mat : nullptr;
  int* nullmask = RANK ? p.nullmask + mat : nullptr;

  __shared__ __attribute__((aligned(16))) float S0[CB * CBP];   // diagonal block / W11
  __shared__ __attribute__((aligned(16))) float S1[CB * CBP];
  __shared__ __attribute__((aligned(16))) float S2[CB * CBP];
  __shared__ float rsv[CB];
  __shared__ volatile int scaled;
  __shared__ volatile int raw_done;
  __shared__ int gave_up;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave & 1, wn = wave >> 1, lr = lane & 31, lk = lane >> 5;
  const int wg = blockIdx.x, a = wg / pc, b = wg % pc;
  // this thread's part of a 64x64 tile in the MFMA result layout: rows frow + 8 (v / 4) + v % 4, column fcol
  const int frow = wm * 32 + 4 * lk, fcol = wn * 32 + lr;
  const int foff = frow * ld + fcol;
  if (t == 0) gave_up = 0;
  __syncthreads();

  int s0_holds = -1;             // panel whose W11 is in S0
  // A tile of L that sits in S1 and still has to be written out and announced; the wave that has nothing
  // to do during the next D does that, off the chain of dependent steps.
  gu64* pending_flag = nullptr;
  gfloat* pending_tile = nullptr;
  u64 pending_value = 0;

  // D(k).  in_lds: the block is already in S0 (lower part, zeros above the diagonal).
  auto do_diag = [&](int k, bool in_lds) __attribute__((always_inline)) {
    const int at = (k * CB) * ld + k * CB;
    if (!in_lds) {
      for (int idx = t; idx < CB * CB / 4; idx += 256) {
        const int rr = idx >> 4, cc = (idx & 15) * 4;
        f32x4_t v = *(const gf32x4*)(x.C + at + rr * ld + cc);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (cc + e > rr) v[e] = 0.f;
        *(f32x4_t*)(S0 + rr * CBP + cc) = v;
      }
    }
    if (t == 0) { scaled = 0; raw_done = 0; }
    __syncthreads();
    if (wave == 0) {
      eliminate_wave<RANK>((lds_float*)S0, (lds_counter*)&raw_done, lane, RANK ? thr + k * CB : nullptr);
    } else if (wave == 2) {
      scale_wave<RANK>((const lds_float*)S0, (lds_counter*)&raw_done, (lds_float*)rsv, (lds_counter*)&scaled, lane, x.piv_lo, x.piv_hi,
                       (float*)(x.L + at), ld, x.status, RANK ? thr + k * CB : nullptr, RANK ? nullmask + k * CB : nullptr);
    } else if (wave == 1) {
      invert_wave<RANK>((lds_float*)S0, (lds_counter*)&raw_done, (const lds_float*)rsv, (lds_counter*)&scaled, lane,
                        RANK ? thr + k * CB : nullptr);
    } else if (pending_flag) {
#pragma unroll 8
      for (int rr = 0; rr < CB; ++rr) shared_store(pending_tile + rr * ld + lane, S1[rr * CBP + lane]);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      if (lane == 0) flag_store(pending_flag, pending_value);
    }
    pending_flag = nullptr;
    __syncthreads();
    lds_to_shared_tile(x.W + at, ld, S0, t);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's stores have completed before the barrier
    __syncthreads();
    if (t == 0) flag_store(x.wflag + k, x.epoch);
    s0_holds = k;
  };

  // T(i, k); leaves L[i][k] in S1 as well.  defer_flag: the flag goes out during the next D
  auto do_column_tile = [&](int i, int k, bool defer_flag) __attribute__((always_inline)) -> bool {
    __syncthreads();   // earlier readers of S0 / S1 are through
    tile_to_lds(S1, x.C + (i * CB) * ld + k * CB, ld, t);
    if (s0_holds != k) {
      if (!wait_until(x, &gave_up, t == 0, [&] { return flag_load(x.wflag + k) == x.epoch; })) return false;
      shared_tile_to_lds(S0, x.W + (k * CB) * ld + k * CB, ld, t);
      s0_holds = k;
    }
    __syncthreads();
    const f32x16_t li = mma_64(S1, S0, wm, wn, lr, lk);   // L[i][k] = C[i][k] W11^T
    __syncthreads();
    gfloat* dst = x.L + (i * CB) * ld + k * CB;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      S1[(frow + 8 * (v / 4) + (v % 4)) * CBP + fcol] = li[v];
      if (!defer_flag) shared_store(dst + foff + (8 * (v / 4) + (v % 4)) * ld, li[v]);
    }
    if (defer_flag) {
      pending_flag = x.lflag + i;
      pending_tile = dst;
      pending_value = (x.epoch << 32) | (u64)(k + 1);
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();   // S1 is complete (and, unless deferred, everybody's stores have completed)
    if (!defer_flag && t == 0) flag_store(x.lflag + i, (x.epoch << 32) | (u64)(k + 1));
    return true;
  };

  // U(i, j, k)
  auto do_update = [&](int i, int j, int k) __attribute__((always_inline)) {
    gfloat* ct = x.C + (i * CB) * ld + j * CB + foff;
    float cold[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) cold[v] = ct[(8 * (v / 4) + (v % 4)) * ld];
    __syncthreads();   // earlier readers of S1 / S2 are through
    shared_tile_to_lds(S1, x.L + (i * CB) * ld + k * CB, ld, t);
    if (j != i) shared_tile_to_lds(S2, x.L + (j * CB) * ld + k * CB, ld, t);
    __syncthreads();
    const f32x16_t up = mma_64(S1, (j != i) ? S2 : S1, wm, wn, lr, lk);
#pragma unroll
    for (int v = 0; v < 16; ++v) ct[(8 * (v / 4) + (v % 4)) * ld] = cold[v] - up[v];
  };

  // U(k1, k1, k1 - 1) with L[k1][k1 - 1] in S1; the result goes straight into S0 for D(k1) and nowhere else
  auto do_update_to_diag = [&](int k1) __attribute__((always_inline)) {
    const gfloat* ct = x.C + (k1 * CB) * ld + k1 * CB + foff;
    float cold[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) cold[v] = ct[(8 * (v / 4) + (v % 4)) * ld];
    const f32x16_t up = mma_64(S1, S1, wm, wn, lr, lk);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = frow + 8 * (v / 4) + (v % 4);
      S0[row * CBP + fcol] = (fcol <= row) ? cold[v] - up[v] : 0.f;
    }
    s0_holds = -1;
  };

  // Step k handles panel k after the diagonal block k+1 has been taken care of (step -1: block 0 only).
  for (int k = -1; k + 1 < nb; ++k) {
    // the chain: T(k+1, k), U(k+1, k+1, k), D(k+1)
    if (((k + 1) % pr) * pc + ((k + 1) % pc) == wg) {
      if (k >= 0) {
        if (!do_column_tile(k + 1, k, true)) return;
        do_update_to_diag(k + 1);
      }
      do_diag(k + 1, k >= 0);
    }
    if (k < 0) continue;
    // the other tiles of column k
    if (k % pc == b) {
      for (int i = a + ((k + 1 - a + pr - 1) / pr) * pr; i < nb; i += pr) {
        if (i <= k || i == k + 1) continue;
        if (!do_column_tile(i, k, false)) return;
      }
    }
    // wait for the tiles of L that this workgroup's updates need: one thread per block row
    {
      bool need = false;
      if (t > k && t < nb) {
        need = (t % pr) == a || (t % pc) == b;   // rows of regular tiles (as i or as j)
        if ((t % pr) * pc + (t % pc) == wg || ((t + 1) < nb && ((t + 1) % pr) * pc + ((t + 1) % pc) == wg)) need = true;   // tiles (i, i-1)
      }
      if (!wait_until(x, &gave_up, need, [&] {
            const u64 v = flag_load(x.lflag + t);
            return (unsigned)(v >> 32) == (unsigned)x.epoch && (unsigned)v >= (unsigned)(k + 1);   // (the tag holds the epoch's low 32 bits)
          }))
        return;
    }
    for (int j = b + ((k + 1 - b + pc - 1) / pc) * pc; j < nb; j += pc) {
      if (j <= k) continue;
      for (int i = a + ((j - a + pr - 1) / pr) * pr; i < nb; i += pr) {
        if (i < j || i == j + 1) continue;
        if (i == j && j == k + 1) continue;   // went into D(k+1) above
        do_update(i, j, k);
      }
    }
    for (int i = k + 2; i < nb; ++i)
      if ((i % pr) * pc + (i % pc) == wg) do_update(i, i - 1, k);
  }
}

// ---------------------------------------------------------------------------------------------------------
// The same factorisation with the chain of dependent steps kept inside ONE workgroup (used when a matrix has sixteen
// workgroups or more to itself).  In the kernel above the chain D(k) -> T(k+1, k) -> U(k+1, k+1, k) -> D(k+1) changes
// workgroups once per panel, and that hand-over (W11 out to memory, a flag, a poll, W11 back in) is about a quarter of
// the panel period.  Here workgroup 0 does nothing but the chain, for all k, with W11 never leaving its LDS on the
// way, and the others ("helpers": pr x pc of them, numbered from 1) do everything else:
//   chain     D(k);  L[k+1][k] = C'[k+1][k] W11^T;  C''[k+1][k+1] = C'[k+1][k+1] - L[k+1][k] L[k+1][k]^T  -> D(k+1)
//   helpers   every other T(i, k) and all updates U(i, j, p) except the last one of a diagonal tile
// where C'[k+1][k] and C'[k+1][k+1] are those two tiles with the updates of all panels before k applied.  Their owner
// (the helper that owns (i, i), (i, i-1) and (i, i-2), so that L[i][i-2] goes from its T task into those two updates
// without leaving LDS) applies the last of them, from panel k-1, before its other work of that panel, and hands the
// tiles to the chain through memory (cflag[k+1]).  That hand-over is off the chain: it happens while the chain
// workgroup factors D(k), whose idle wave polls the flag and fetches the two tiles into LDS.  W11 and L[k+1][k] go out
// to the helpers likewise without the chain waiting for anything but its own stores.
// Tiles that cross between workgroups, the two kinds of look-ahead tile included, are only ever written and read with
// device-scope accesses.  Waits are bounded as above.
//
// FUSE_INV: the helpers also form W = L^-1, row by row behind the factorisation, so that no separate pass over L
// follows it.  With W'(j, e) the running value of tile (j, e), e < j, that starts at zero,
//   UW(j, e, p)  W'(j, e) -= L[j][p] W(p, e)        for e <= p < j        (needs lflag[j] > p and row p of W)
//   TW(p, e)     W(p, e) = W11(p) W'(p, e)           once UW(p, e, p - 1) is through   -> vflag[p][e]
// and W(p, p) = W11(p) as the chain leaves it (wflag[p]; the last one is announced when the chain ends).  Tile (j, e)
// belongs to helper (j mod pr) pc + (e mod pc), which applies UW(j, e, p) for j >= p + 2 after the look-ahead work of
// panel p + 1 (before it, the chain found its next tiles 3 us late) and UW(p + 1, e, p) right before TW(p + 1, e),
// also in panel p + 1: a helper only ever waits for tiles of row p of W while it works on panel p + 1, and their
// owners produce them from flags of the chain and of row p - 1 alone, so the order of the factorisation's own tasks
// is untouched.  Running values are the owner's private data (ordinary accesses); finished tiles are written and
// read with device-scope accesses like the tiles of L.
template <bool RANK, bool FUSE_INV>
__global__ void __launch_bounds__(256, 1) chol_chain_kernel(CholStreamArgs p) {
  const long long mat = (long long)blockIdx.y * p.stride;
  if (p.skip && p.skip[mat] != 0) return;   // uniform for the whole grid row of this matrix
  const int nb = p.rp / CB, pr = p.pr, pc = p.pc;
  StreamCtx x;
  x.C = (gfloat*)(p.C + mat);
  x.L = (gfloat*)(p.L + mat);
  x.W = (gfloat*)(p.W + mat);
  x.status = p.status + blockIdx.y;
  x.wflag = (gu64*)(p.sync + (long long)blockIdx.y * p.sync_stride);
  x.lflag = x.wflag + nb;
  gu64* const cflag = x.lflag + nb;
  x.abort_word = cflag + nb;
  gu64* const vflag = x.wflag + p.vflag_off;   // FUSE_INV: nb x nb words, [p][e] = tile (p, e) of W is final
  x.epoch = *p.step_counter * 8ull + (u64)p.pass;
  x.spin_limit = p.spin_limit;
  x.ld = p.rp;
  x.piv_lo = p.piv_lo;
  x.piv_hi = p.piv_hi;
  const int ld = p.rp;
  const float* thr = RANK ? p.thr + mat : nullptr;
  int* nullmask = RANK ? p.nullmask + mat : nullptr;

  __shared__ __attribute__((aligned(16))) float S0[CB * CBP];   // diagonal block / W11
  __shared__ __attribute__((aligned(16))) float S1[CB * CBP];
  __shared__ __attribute__((aligned(16))) float S2[CB * CBP];
  __shared__ __attribute__((aligned(16))) float S3[CB * CBP];
  __shared__ float rsv[CB];
  __shared__ volatile int scaled;
  __shared__ volatile int raw_done;
  __shared__ int gave_up;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave & 1, wn = wave >> 1, lr = lane & 31, lk = lane >> 5;
  const int frow = wm * 32 + 4 * lk, fcol = wn * 32 + lr;
  const int foff = frow * ld + fcol;
  if (t == 0) gave_up = 0;
  __syncthreads();
  const u64 ep32 = x.epoch << 32;
  auto tile_at = [&](gfloat* base, int i, int j) __attribute__((always_inline)) { return base + (i * CB) * ld + j * CB; };

  if (blockIdx.x == 0) {
    // ---------------------------------------------------------------- the chain
    // diagonal tile 0 (lower part, zeros above the diagonal)
    for (int idx = t; idx < CB * CB / 4; idx += 256) {
      const int rr = idx >> 4, cc = (idx & 15) * 4;
      f32x4_t v = *(const gf32x4*)(x.C + rr * ld + cc);
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (cc + e > rr) v[e] = 0.f;
      *(f32x4_t*)(S0 + rr * CBP + cc) = v;
    }
    for (int k = 0; k < nb; ++k) {
      const int at = (k * CB) * ld + k * CB;
      if (t == 0) { scaled = 0; raw_done = 0; }
      __syncthreads();   // (also: everybody's stores of the last step, W11(k-1) and L[k][k-1], have completed)
#ifdef DION_CHOL_TIMING
      if (t == 0 && p.dbg) p.dbg[8 * k + 0] = wall_clock64();
#endif
      if (t == 0 && k >= 1) {
        flag_store(x.wflag + k - 1, x.epoch);           // W11(k-1) is out, and so is L[k][k-1]:
        flag_store(x.lflag + k, ep32 | (u64)k);         // the helper of the next look-ahead row fetches both at once
      }
      if (wave == 0) {
        eliminate_wave<RANK>((lds_float*)S0, (lds_counter*)&raw_done, lane, RANK ? thr + k * CB : nullptr);
      } else if (wave == 2) {
        scale_wave<RANK>((const lds_float*)S0, (lds_counter*)&raw_done, (lds_float*)rsv, (lds_counter*)&scaled, lane, x.piv_lo, x.piv_hi,
                         (float*)(x.L + at), ld, x.status, RANK ? thr + k * CB : nullptr, RANK ? nullmask + k * CB : nullptr);
      } else if (wave == 1) {
        invert_wave<RANK>((lds_float*)S0, (lds_counter*)&raw_done, (const lds_float*)rsv, (lds_counter*)&scaled, lane,
                          RANK ? thr + k * CB : nullptr);
      } else if (k + 1 < nb) {
        // the idle wave: the two tiles of the next step in, once their owner has applied their last update
        bool ok = true;
#ifdef DION_CHOL_TIMING
        if (lane == 0 && p.dbg) p.dbg[8 * k + 3] = wall_clock64();
#endif
        if (k >= 1) {   // (the tiles of row 1 have no update before panel 0: nothing to wait for)
          unsigned n = 0;
          while (flag_load(cflag + k + 1) != x.epoch) {
            __builtin_amdgcn_s_sleep(1);
            if (++n > x.spin_limit) {
              flag_store(x.abort_word, x.epoch);
              if (*x.status == 0) *x.status = ST_TIMEOUT;
              *(volatile int*)&gave_up = 1;
              ok = false;
              break;
            }
            if ((n & 31u) == 0 && flag_load(x.abort_word) == x.epoch) {
              *(volatile int*)&gave_up = 1;
              ok = false;
              break;
            }
          }
        }
#ifdef DION_CHOL_TIMING
        if (lane == 0 && p.dbg) p.dbg[8 * k + 4] = wall_clock64();
#endif
        if (ok) {
          const gfloat* sub = tile_at(x.C, k + 1, k);
          const gfloat* dia = tile_at(x.C, k + 1, k + 1);
          // (all loads of both tiles are issued before the first of them is waited for: one memory round trip)
          float a[CB], d[CB];
#pragma unroll
          for (int rr = 0; rr < CB; ++rr) a[rr] = shared_load(sub + rr * ld + lane);
#pragma unroll
          for (int rr = 0; rr < CB; ++rr) d[rr] = shared_load(dia + rr * ld + lane);
#pragma unroll
          for (int rr = 0; rr < CB; ++rr) S2[rr * CBP + lane] = a[rr];
#pragma unroll
          for (int rr = 0; rr < CB; ++rr) S3[rr * CBP + lane] = d[rr];
#ifdef DION_CHOL_TIMING
          if (lane == 0 && p.dbg) p.dbg[8 * k + 5] = wall_clock64();
#endif
        }
      }
      __syncthreads();
#ifdef DION_CHOL_TIMING
      if (t == 0 && p.dbg) p.dbg[8 * k + 1] = wall_clock64();
#endif
      if (*(volatile int*)&gave_up) return;   // uniform: written before the barrier
      // W11 out to the helpers; nobody here waits for these stores before the step is through
      lds_to_shared_tile(x.W + at, ld, S0, t);
      if (k + 1 == nb) {
        if (FUSE_INV) {   // the last row of W waits for this W11
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          __syncthreads();
          if (t == 0) flag_store(x.wflag + k, x.epoch);
        }
        break;
      }
      const f32x16_t li = mma_64(S2, S0, wm, wn, lr, lk);   // L[k+1][k] = C'[k+1][k] W11^T
      gfloat* dst = tile_at(x.L, k + 1, k);
#pragma unroll
      for (int v = 0; v < 16; ++v) shared_store(dst + foff + (8 * (v / 4) + (v % 4)) * ld, li[v]);
      __syncthreads();                                      // everybody has read S0 and S2
#pragma unroll
      for (int v = 0; v < 16; ++v) S1[(frow + 8 * (v / 4) + (v % 4)) * CBP + fcol] = li[v];
      __syncthreads();
      const f32x16_t up = mma_64(S1, S1, wm, wn, lr, lk);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = frow + 8 * (v / 4) + (v % 4);
        S0[row * CBP + fcol] = (fcol <= row) ? S3[row * CBP + fcol] - up[v] : 0.f;
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // this thread's parts of W11(k) and L[k+1][k] are in memory
#ifdef DION_CHOL_TIMING
      if (t == 0 && p.dbg) p.dbg[8 * k + 2] = wall_clock64();
#endif
    }
    return;
  }

  // ------------------------------------------------------------------ a helper
  // Ownership: the tiles (i, i), (i, i-1), (i, i-2) of a row i go together, to helper (i mod pr) pc + (i mod pc); any
  // other tile (i, j) to helper (i mod pr) pc + (j mod pc).  With pr and pc coprime the rows of the first kind that a
  // helper owns are i0, i0 + pr pc, ...
  const int h = (int)blockIdx.x - 1, a = h / pc, b = h % pc;
  int i0 = -1;
  for (int i = a; i < pr * pc; i += pr)
    if (i % pc == b) { i0 = i; break; }
  const int istep = pr * pc;
  auto owns_row = [&](int i) __attribute__((always_inline)) { return i0 >= 0 && i >= i0 && (i - i0) % istep == 0; };
  int s0_holds = -1;   // panel whose W11 is in S0
  // T(i, p): L[i][p] = C[i][p] W11(p)^T, published; leaves it in S1 as well
  auto column_tile = [&](int i, int p_) __attribute__((always_inline)) -> bool {
    __syncthreads();   // earlier readers of S0 / S1 are through
    tile_to_lds(S1, tile_at(x.C, i, p_), ld, t);
    if (s0_holds != p_) {
      if (!wait_until(x, &gave_up, t == 0, [&] { return flag_load(x.wflag + p_) == x.epoch; })) return false;
      shared_tile_to_lds(S0, tile_at(x.W, p_, p_), ld, t);
      s0_holds = p_;
    }
    __syncthreads();
    const f32x16_t li = mma_64(S1, S0, wm, wn, lr, lk);
    __syncthreads();
    gfloat* dst = tile_at(x.L, i, p_);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      S1[(frow + 8 * (v / 4) + (v % 4)) * CBP + fcol] = li[v];
      shared_store(dst + foff + (8 * (v / 4) + (v % 4)) * ld, li[v]);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();   // S1 is complete, everybody's stores have completed
    if (t == 0) flag_store(x.lflag + i, ep32 | (u64)(p_ + 1));
    return true;
  };
  // U(i, j, p): C[i][j] -= L[i][p] L[j][p]^T.  li_in_s1: L[i][p] is in S1 already.  shared: the tile is of the kind that
  // ends up with the chain (diagonal and first sub-diagonal): device-scope accesses throughout.
  auto update = [&](int i, int j, int p_, bool li_in_s1, bool shared) __attribute__((always_inline)) {
    gfloat* ct = tile_at(x.C, i, j) + foff;
    float cold[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) cold[v] = shared ? shared_load(ct + (8 * (v / 4) + (v % 4)) * ld) : ct[(8 * (v / 4) + (v % 4)) * ld];
    // (all three tiles are requested before the first wait: one memory round trip per update, not three)
    float li[16], lj[16];
    if (!li_in_s1) shared_tile_to_regs(li, tile_at(x.L, i, p_), ld, t);
    if (j != i) shared_tile_to_regs(lj, tile_at(x.L, j, p_), ld, t);
    __syncthreads();   // earlier readers of S1 / S2 are through
    if (!li_in_s1) regs_to_lds<false>(S1, li, t);
    if (j != i) regs_to_lds<false>(S2, lj, t);
    __syncthreads();
    const f32x16_t up = mma_64(S1, (j != i) ? S2 : S1, wm, wn, lr, lk);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      if (shared) shared_store(ct + (8 * (v / 4) + (v % 4)) * ld, cold[v] - up[v]);
      else ct[(8 * (v / 4) + (v % 4)) * ld] = cold[v] - up[v];
    }
  };
  auto row_ready = [&](int row, int cols) __attribute__((always_inline)) {   // L[row][0 .. cols) are out
    const u64 v = flag_load(x.lflag + row);
    return (unsigned)(v >> 32) == (unsigned)x.epoch && (unsigned)v >= (unsigned)cols;
  };
  // ---- the inverse (FUSE_INV)
  auto w_ready = [&](int p_, int e) __attribute__((always_inline)) {   // tile (p_, e) of W is final
    return flag_load(e == p_ ? x.wflag + p_ : vflag + p_ * nb + e) == x.epoch;
  };
  // UW(j, e, p): W'(j, e) -= L[j][p] W(p, e); the first one, p = e, starts from zero
  auto w_update = [&](int j, int e, int p_) __attribute__((always_inline)) {
    gfloat* wt = tile_at(x.W, j, e) + foff;
    float cold[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) cold[v] = p_ > e ? wt[(8 * (v / 4) + (v % 4)) * ld] : 0.f;
    float lj[16], wp[16];
    shared_tile_to_regs(lj, tile_at(x.L, j, p_), ld, t);
    shared_tile_to_regs(wp, tile_at(x.W, p_, e), ld, t);
    __syncthreads();   // earlier readers of S1 / S2 are through
    regs_to_lds<false>(S1, lj, t);
    regs_to_lds<true>(S2, wp, t);
    __syncthreads();
    const f32x16_t up = mma_64(S1, S2, wm, wn, lr, lk);   // L[j][p] (W(p, e)^T)^T
#pragma unroll
    for (int v = 0; v < 16; ++v) wt[(8 * (v / 4) + (v % 4)) * ld] = cold[v] - up[v];
  };
  // Row p_ of W into the running values of the rows from p_ + 2 down that this helper has tiles in (L[j][p_] is out:
  // the wait before the updates of panel p_ covers the rows j = a mod pr)
  auto w_rest = [&](int p_) __attribute__((always_inline)) -> bool {
    const int j0 = a + ((p_ + 2 - a + pr - 1) / pr) * pr;
    if (j0 >= nb || b > p_) return true;   // (uniform)
    if (!wait_until(x, &gave_up, t <= p_ && t % pc == b, [&] { return w_ready(p_, t); })) return false;
    for (int j = j0; j < nb; j += pr)
      for (int e = b; e <= p_; e += pc) w_update(j, e, p_);
    return true;
  };
  // Row p_ of W, for the tiles of it that this helper owns: their last update, then W(p_, e) = W11(p_) W'(p_, e)
  auto w_row = [&](int p_) __attribute__((always_inline)) -> bool {
    if (p_ < 1 || p_ % pr != a || b > p_ - 1) return true;   // (uniform)
    if (!wait_until(x, &gave_up, t < p_ && t % pc == b, [&] { return w_ready(p_ - 1, t); })) return false;
    if (!wait_until(x, &gave_up, t == 0, [&] { return row_ready(p_, p_); })) return false;
    for (int e = b; e < p_; e += pc) w_update(p_, e, p_ - 1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's parts of the running values are in memory
    for (int e = b; e < p_; e += pc) {
      gfloat* wt = tile_at(x.W, p_, e) + foff;
      float run[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) run[v] = wt[(8 * (v / 4) + (v % 4)) * ld];
      __syncthreads();   // earlier readers of S0 / S1 are through
#pragma unroll
      for (int v = 0; v < 16; ++v) S1[fcol * CBP + frow + 8 * (v / 4) + (v % 4)] = run[v];   // W'(p_, e)^T
      if (s0_holds != p_) {
        if (!wait_until(x, &gave_up, t == 0, [&] { return flag_load(x.wflag + p_) == x.epoch; })) return false;
        shared_tile_to_lds(S0, tile_at(x.W, p_, p_), ld, t);
        s0_holds = p_;
      }
      __syncthreads();
      const f32x16_t res = mma_64(S0, S1, wm, wn, lr, lk);   // W11(p_) W'(p_, e)
#pragma unroll
      for (int v = 0; v < 16; ++v) shared_store(wt + (8 * (v / 4) + (v % 4)) * ld, res[v]);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();   // everybody's stores have completed
      if (t == 0) flag_store(vflag + p_ * nb + e, x.epoch);
    }
    return true;
  };

  for (int p_ = 0; p_ + 1 < nb; ++p_) {
    // Row p_ + 2 feeds the chain's next step: its owner turns (p_ + 2, p_) into a tile of L first and applies that
    // row's two look-ahead updates at once, before anything else of this panel.
    if (p_ + 2 < nb && owns_row(p_ + 2)) {
      // (Everything that does not depend on W11(p_) is fetched before the wait for it, results are stored without
      // waiting in between, and one wait for all stores comes before the flags: this path decides whether the chain
      // finds its tiles ready when it has factored its diagonal block.)
      const int i = p_ + 2;
      __syncthreads();   // earlier readers of S0 / S1 / S2 are through
      tile_to_lds(S1, tile_at(x.C, i, p_), ld, t);
      gfloat* cd = tile_at(x.C, i, i) + foff;
      gfloat* cs = tile_at(x.C, i, i - 1) + foff;
      float cold_d[16], cold_s[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        cold_d[v] = shared_load(cd + (8 * (v / 4) + (v % 4)) * ld);
        cold_s[v] = shared_load(cs + (8 * (v / 4) + (v % 4)) * ld);
      }
      // (the chain announces W11(p_) once L[p_+1][p_] is out as well: one wait, both tiles in one go)
      if (!wait_until(x, &gave_up, t == 0, [&] { return flag_load(x.wflag + p_) == x.epoch; })) return;
      shared_tile_to_lds(S0, tile_at(x.W, p_, p_), ld, t);
      shared_tile_to_lds(S2, tile_at(x.L, p_ + 1, p_), ld, t);
      s0_holds = p_;
      __syncthreads();
      const f32x16_t li = mma_64(S1, S0, wm, wn, lr, lk);   // L[i][p_]
      __syncthreads();
      gfloat* dst = tile_at(x.L, i, p_);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        S1[(frow + 8 * (v / 4) + (v % 4)) * CBP + fcol] = li[v];
        shared_store(dst + foff + (8 * (v / 4) + (v % 4)) * ld, li[v]);
      }
      __syncthreads();   // S1 is complete
      const f32x16_t upd = mma_64(S1, S1, wm, wn, lr, lk);
#pragma unroll
      for (int v = 0; v < 16; ++v) shared_store(cd + (8 * (v / 4) + (v % 4)) * ld, cold_d[v] - upd[v]);
      const f32x16_t ups = mma_64(S1, S2, wm, wn, lr, lk);
#pragma unroll
      for (int v = 0; v < 16; ++v) shared_store(cs + (8 * (v / 4) + (v % 4)) * ld, cold_s[v] - ups[v]);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();   // everybody's stores (L[i][p_] and the two updated tiles) have completed
      if (t == 0) {
        flag_store(cflag + i, x.epoch);   // both tiles of row i carry all updates up to panel i - 2
        flag_store(x.lflag + i, ep32 | (u64)(p_ + 1));
      }
    }
    // the other tiles of column p_ that this helper turns into tiles of L (three rows below the diagonal and further)
    if (p_ % pc == b)
      for (int i = a + ((p_ + 3 - a + pr - 1) / pr) * pr; i < nb; i += pr)
        if (!column_tile(i, p_)) return;
    // the inverse: row p_ - 1 of W into the rows from p_ + 1 down (kept until now so that it does not stand between
    // the previous panel and this one's look-ahead work), then this helper's part of row p_
    if (FUSE_INV && p_ >= 1 && !w_rest(p_ - 1)) return;
    if (FUSE_INV && !w_row(p_)) return;
    // the tiles of L that this helper's other updates of panel p_ need: one thread per block row (a superset)
    {
      bool need = false;
      if (t > p_ && t < nb) need = (t % pr) == a || (t % pc) == b || owns_row(t) || owns_row(t + 1) || owns_row(t + 2);
      if (!wait_until(x, &gave_up, need, [&] { return row_ready(t, p_ + 1); })) return;
    }
    // updates of the tiles three and more below the diagonal
    for (int j = b + ((p_ + 1 - b + pc - 1) / pc) * pc; j < nb; j += pc)
      for (int i = a + ((j + 3 - a + pr - 1) / pr) * pr; i < nb; i += pr) update(i, j, p_, false, false);
    // ... and of the rows whose near-diagonal tiles are this helper's (row p_ + 2 was done above; the last update of a
    // diagonal tile, from the panel just left of it, is the chain's)
    if (i0 >= 0)
      for (int i = i0; i < nb; i += istep) {
        if (i < p_ + 3) continue;
        update(i, i, p_, false, true);
        update(i, i - 1, p_, false, true);
        update(i, i - 2, p_, false, false);
      }
  }
  if (FUSE_INV) w_row(nb - 1);   // (row nb - 2 of W has no rows from nb down to go into)
}

hipError_t launch_chol_stream(CholStreamArgs p, int batch, hipStream_t s) {
  // 32 KB of unused dynamic LDS on top of the 52 KB the kernel declares: one workgroup per compute unit, so the
  // workgroup on the critical chain shares its unit with nobody
  if (p.chain) {
    // (70 KB of declared LDS and 32 KB of unused dynamic LDS: more than half of a compute unit's, so one workgroup each)
    // (the inverse needs a flag word per tile of W, and its waits one thread per panel; measured up to 64 panels)
    if (p.vflag_off > 0 && (p.thr || p.rp / CB > FUSED_INV_MAX_NB)) return hipErrorInvalidValue;
    if (p.thr) hipLaunchKernelGGL((chol_chain_kernel<true, false>), dim3(p.pr * p.pc + 1, batch), dim3(256), 32768, s, p);
    else if (p.vflag_off > 0) hipLaunchKernelGGL((chol_chain_kernel<false, true>), dim3(p.pr * p.pc + 1, batch), dim3(256), 32768, s, p);
    else hipLaunchKernelGGL((chol_chain_kernel<false, false>), dim3(p.pr * p.pc + 1, batch), dim3(256), 32768, s, p);
    return hipGetLastError();
  }
  if (p.thr) hipLaunchKernelGGL(chol_stream_kernel<true>, dim3(p.pr * p.pc, batch), dim3(256), 32768, s, p);
  else hipLaunchKernelGGL(chol_stream_kernel<false>, dim3(p.pr * p.pc, batch), dim3(256), 32768, s, p);
  return hipGetLastError();
}

hipError_t launch_chol_panel(CholPanelPtrs p, int batch, int k0, int rp, float piv_lo, float piv_hi, hipStream_t s) {
  const int nb = (rp - k0 - CB) / CB;
  const int tiles = nb * (nb + 1) / 2;
  auto go = [&](int blocks, int mode) {
    if (p.thr) hipLaunchKernelGGL(chol_panel_kernel<true>, dim3(blocks, batch), dim3(256), 0, s, p, k0, rp, piv_lo, piv_hi, mode);
    else hipLaunchKernelGGL(chol_panel_kernel<false>, dim3(blocks, batch), dim3(256), 0, s, p, k0, rp, piv_lo, piv_hi, mode);
    return hipGetLastError();
  };
  if ((long long)(1 + tiles) * batch <= 1024 || tiles == 0) return go(1 + tiles, 0);
  hipError_t e = go(1, 1);
  if (e != hipSuccess) return e;
  return go(tiles, 2);
}

}  // namespace dion
