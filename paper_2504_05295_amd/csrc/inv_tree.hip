// W = L^-1 for the r x r Cholesky factor of Cholesky-QR (Appendix A), in one launch.
//
// The factorisation leaves L and the inverses of its 64 x 64 diagonal blocks.  Neighbouring diagonal blocks
// are merged level by level,
//     [[A, 0], [C, D]]^-1 = [[A^-1, 0], [-D^-1 C A^-1, D^-1]],
// at level l blocks of 64 * 2^l (the last one may be shorter; a block without a right-hand neighbour waits for
// the next level).  A merge is two products of triangular with full matrices, T = C A^-1 and then -D^-1 T,
// cut into 64 x 64 output tiles that skip the zero tiles of the triangular operand; the tiles of all merges
// of a level are dealt out to the workgroups of the matrix by length, so that each gets about the same work.
// Between the two products, and between levels, the workgroups of a matrix meet at a barrier made of one arrival
// word per workgroup (tagged with the launch's epoch, so never cleared); what crosses between workgroups is
// written and read with device-scope accesses.
// Waits are bounded as in the factorisation kernel: who gives up raises the abort word, the others follow,
// and the matrix is reported with the wait-timeout status.  All workgroups of a launch must be resident at once (the host keeps
// the grid within one workgroup per compute unit).
#include <type_traits>

#include "internal.hpp"
#include "inv_tree_order.hpp"

namespace dion {

namespace {
typedef unsigned long long u64;
typedef __attribute__((address_space(1))) u64 gu64;
typedef __attribute__((address_space(1))) float gfloat;
typedef __attribute__((address_space(1))) int gint;
constexpr int CB = CHOL_NB;   // 64
constexpr int CBP = CB + 4;   // LDS row stride (floats): conflict-free 16-byte reads
constexpr int DEPTH = 3;      // tile pairs in flight per workgroup

__device__ __forceinline__ u64 flag_load(const gu64* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void flag_store(gu64* p, u64 v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
// Tiles written in this launch (T, the merged parts of W) cross between workgroups: they are written and read with
// device-scope accesses, which go past the caches private to a compute unit or to one part of the chip, so that no
// cache-wide write-back or invalidation is needed, only that a writer's stores have completed before it arrives at
// the barrier.
__device__ __forceinline__ float shared_load(const gfloat* p) {
  return __int_as_float(__hip_atomic_load((const gint*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void shared_store(gfloat* p, float v) {
  __hip_atomic_store((gint*)p, __float_as_int(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

struct TreeCtx {
  gu64* arrive;       // one word per workgroup of this matrix
  gu64* abort_word;
  int* status;
  u64 epoch;
  unsigned spin_limit;
  int groups, wg;
};

// All workgroups of the matrix have arrived, and what they stored before is in memory.  Returns false (for all
// threads) when a wait was given up, here or elsewhere.
__device__ __forceinline__ bool group_barrier(const TreeCtx& x, unsigned& count, int* gave_up, int t) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's stores have completed
  __syncthreads();
  ++count;
  if (t == 0) flag_store(x.arrive + x.wg, (x.epoch << 32) | (u64)count);
  if (t < x.groups) {
    unsigned n = 0;
    for (;;) {
      const u64 v = flag_load(x.arrive + t);
      if ((unsigned)(v >> 32) == (unsigned)x.epoch && (unsigned)v >= count) break;   // (the tag holds the epoch's low 32 bits)
      __builtin_amdgcn_s_sleep(1);
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

// This thread's share of two 64 x 64 fp32 tiles (row-major in memory): column t % 64 of rows t / 64 + 4 e.
struct TilePair {
  float a[16], b[16];
};
// A_SHARED: the left tile was written in this launch too (else it comes from the factorisation: ordinary loads)
// (A and B are uniform tile addresses; offs holds this thread's 16 element offsets within a tile)
template <bool A_SHARED>
__device__ __forceinline__ void fetch(TilePair& r, const float* A, const float* B, const unsigned (&offs)[16]) {
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    r.a[e] = A_SHARED ? shared_load((const gfloat*)A + offs[e]) : A[offs[e]];
    r.b[e] = shared_load((const gfloat*)B + offs[e]);
  }
}
// As[m][k] and Bs[k][n], both as they are in memory
__device__ __forceinline__ void stash(const TilePair& r, float* As, float* Bs, int t) {
  const int r0 = t >> 6, c = t & 63;
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    As[(r0 + 4 * e) * CBP + c] = r.a[e];
    Bs[(r0 + 4 * e) * CBP + c] = r.b[e];
  }
}
// acc += As[64 x 64] * Bs[64 x 64] for this wave's 32 x 32 quadrant
__device__ __forceinline__ void mma_tile(f32x16_t& acc, const float* As, const float* Bs, int wm, int wn, int lr, int lk) {
#pragma unroll
  for (int kk = 0; kk < CB; kk += 8) {
    const f32x4_t a = *(const f32x4_t*)(As + (wm * 32 + lr) * CBP + kk + lk * 4);
    float b[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) b[s] = Bs[(kk + lk * 4 + s) * CBP + wn * 32 + lr];
#pragma unroll
    for (int s = 0; s < 4; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], b[s], acc, 0, 0, 0);
  }
}
}  // namespace

__global__ void __launch_bounds__(256) inv_tree_kernel(InvTreeArgs p) {
  const long long mat = (long long)blockIdx.y * p.stride;
  if (p.skip && p.skip[mat] != 0) return;   // uniform for all workgroups of this matrix
  const int nb = p.rp / CB, ld = p.rp;
  const float* L = p.L + mat;
  float* W = p.W + mat;
  float* T = p.T + mat;
  TreeCtx x;
  x.arrive = (gu64*)(p.sync + (long long)blockIdx.y * p.sync_stride);
  x.abort_word = x.arrive + INV_TREE_MAX_GROUPS;
  x.status = p.status + blockIdx.y;
  x.epoch = *p.step_counter * 8ull + (u64)p.pass;
  x.spin_limit = p.spin_limit;
  x.groups = gridDim.x;
  x.wg = blockIdx.x;

  __shared__ __attribute__((aligned(16))) float As[CB * CBP];
  __shared__ __attribute__((aligned(16))) float Bs[CB * CBP];
  __shared__ int gave_up;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave & 1, wn = wave >> 1, lr = lane & 31, lk = lane >> 5;
  // this thread's part of a 64 x 64 tile in the MFMA result layout: rows frow + 8 (v / 4) + v % 4, column fcol
  const int frow = wm * 32 + 4 * lk, fcol = wn * 32 + lr;
  if (t == 0) gave_up = 0;
  __syncthreads();
  unsigned barriers = 0;
  unsigned offs[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) offs[e] = (unsigned)(((t >> 6) + 4 * e) * ld + (t & 63));

  // out tile = sign * sum over k in [k_lo, k_hi] of Atile(k) Btile(k), with Atile(k) = tile (a_row, a_col0 + k) of Amat
  // and Btile(k) = tile (b_row0 + k, b_col) of Bmat (tile coordinates in units of 64).  DEPTH tile pairs are kept in
  // flight: a pair costs two memory round trips' worth of latency and about a third of that in matrix instructions.
  auto product = [&](auto a_shared, const float* Amat, int a_row, int a_col0, const float* Bmat, int b_row0, int b_col, int k_lo,
                     int k_hi, float* out, float sign) __attribute__((always_inline)) {
    constexpr bool AS = decltype(a_shared)::value;
    f32x16_t acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    const float* Ap = Amat + ((long long)a_row * ld + a_col0) * CB;   // + k * CB
    const float* Bp = Bmat + ((long long)b_row0 * ld + b_col) * CB;   // + k * ld * CB
    TilePair regs[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
      if (k_lo + d <= k_hi) fetch<AS>(regs[d], Ap + (long long)(k_lo + d) * CB, Bp + (long long)(k_lo + d) * ld * CB, offs);
    for (int k = k_lo; k <= k_hi; k += DEPTH) {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        if (k + d <= k_hi) {
          __syncthreads();   // the previous pair's reads of As / Bs are through
          stash(regs[d], As, Bs, t);
          if (k + d + DEPTH <= k_hi)
            fetch<AS>(regs[d], Ap + (long long)(k + d + DEPTH) * CB, Bp + (long long)(k + d + DEPTH) * ld * CB, offs);
          __syncthreads();
          mma_tile(acc, As, Bs, wm, wn, lr, lk);
        }
      }
    }
    gfloat* o = (gfloat*)out + (long long)frow * ld + fcol;
#pragma unroll
    for (int v = 0; v < 16; ++v) shared_store(o + (long long)(8 * (v / 4) + (v % 4)) * ld, sign * acc[v]);
  };

  for (int S = 1; S < nb; S *= 2) {
    const int rounds = inv_tree_rounds(nb, S, x.groups);
    for (int phase = 0; phase < 2; ++phase) {
      for (int round = 0; round < rounds; ++round) {
        int q, ti, tj;
        if (!inv_tree_tile(nb, S, phase, x.groups, x.wg, round, q, ti, tj)) continue;
        const int a0 = 2 * q * S, d0 = a0 + S;
        if (phase == 0) {
          // T[d0+ti][a0+tj] = sum_{k=tj}^{S-1} L[d0+ti][a0+k] W[a0+k][a0+tj]      (A^-1 is lower triangular)
          product(std::false_type{}, L, d0 + ti, a0, W, a0, a0 + tj, tj, S - 1, T + ((long long)(d0 + ti) * ld + (a0 + tj)) * CB, 1.f);
        } else {
          // W[d0+ti][a0+tj] = -sum_{k=0}^{ti} W[d0+ti][d0+k] T[d0+k][a0+tj]      (D^-1 is lower triangular)
          product(std::true_type{}, W, d0 + ti, d0, T, d0, a0 + tj, 0, ti, W + ((long long)(d0 + ti) * ld + (a0 + tj)) * CB, -1.f);
        }
      }
      if (phase == 1 && 2 * S >= nb) break;   // nobody reads the last level's result in this launch
      if (!group_barrier(x, barriers, &gave_up, t)) return;
    }
  }
}

hipError_t launch_inv_tree(InvTreeArgs p, int groups, int batch, int cus, hipStream_t s) {
  if (groups < 1 || groups > INV_TREE_MAX_GROUPS || (long long)groups * batch > cus) return hipErrorInvalidValue;
  hipLaunchKernelGGL(inv_tree_kernel, dim3(groups, batch), dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace dion
