// Element-wise, reduction and panel kernels of the Dion step (everything that is not a tiled GEMM).
#include "internal.hpp"

namespace dion {

// ---------------------------------------------------------------- pointer table refresh
struct UserPtrChunk {
  void* p[48][4];
  int first_row, count, nslots;
};
// status != nullptr: the status words of these rows are cleared as well.  counter != nullptr: that 64-bit word is
// incremented (once per step: the single-launch Cholesky kernel tags its flags with it).
__global__ void set_user_ptrs_kernel(void** table, const UserPtrChunk c, int* status, unsigned long long* counter) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t == 0 && counter) *counter += 1ull;
  if (status && t < c.count) status[c.first_row + t] = 0;
  if (t >= c.count * 4) return;
  table[(size_t)(c.first_row + t / 4) * c.nslots + (t % 4)] = c.p[t / 4][t % 4];
}
hipError_t launch_set_user_ptrs(void** table, int nslots, int first_row, int count, void* const* X, const void* const* G,
                                void* const* M, void* const* Q, hipStream_t s, int* status, unsigned long long* counter) {
  for (int done = 0; done < count; done += 48) {
    UserPtrChunk c;
    c.first_row = first_row + done;
    c.count = (count - done < 48) ? count - done : 48;
    c.nslots = nslots;
    for (int i = 0; i < c.count; ++i) {
      c.p[i][SLOT_X] = X[done + i];
      c.p[i][SLOT_G] = const_cast<void*>(G[done + i]);
      c.p[i][SLOT_M] = M[done + i];
      c.p[i][SLOT_Q] = Q[done + i];
    }
    hipLaunchKernelGGL(set_user_ptrs_kernel, dim3(1), dim3(256), 0, s, table, c, status, done == 0 ? counter : nullptr);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// One whole row of the pointer table from kernel arguments (a state whose table cannot be written with a host copy:
// the call may be part of a stream capture); also copies an int32 from *src to *dst when both are given.
struct TableRow {
  void* p[NSLOTS];
};
__global__ void set_table_row_kernel(void** table, const TableRow row) {
  if (threadIdx.x < NSLOTS) table[threadIdx.x] = row.p[threadIdx.x];
}
hipError_t launch_set_table_row(void** table, void* const* values, hipStream_t s) {
  TableRow row;
  for (int i = 0; i < NSLOTS; ++i) row.p[i] = values[i];
  hipLaunchKernelGGL(set_table_row_kernel, dim3(1), dim3(64), 0, s, table, row);
  return hipGetLastError();
}
__global__ void copy_i32_kernel(const int* src, int* dst) {
  if (threadIdx.x == 0) *dst = *src;
}
hipError_t launch_copy_i32(const int* src, int* dst, hipStream_t s) {
  hipLaunchKernelGGL(copy_i32_kernel, dim3(1), dim3(64), 0, s, src, dst);
  return hipGetLastError();
}

// status[dst_row[i]] = other_status[src_row[i]]: the second stage of a Double Dion step starts from the outcome of the
// first (a matrix that failed there is skipped here as well)
struct RowPairChunk {
  int src[96], dst[96];
  int count;
};
__global__ void copy_status_rows_kernel(const int* src_status, int* dst_status, const RowPairChunk c) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < c.count) dst_status[c.dst[t]] = src_status[c.src[t]] != 0 ? ST_UPSTREAM : ST_OK;   // failed before this stage began
}
hipError_t launch_copy_status_rows(const int* src_status, int* dst_status, int count, const int* src_rows, const int* dst_rows,
                                   hipStream_t s) {
  for (int done = 0; done < count; done += 96) {
    RowPairChunk c;
    c.count = (count - done < 96) ? count - done : 96;
    for (int i = 0; i < c.count; ++i) { c.src[i] = src_rows[done + i]; c.dst[i] = dst_rows[done + i]; }
    hipLaunchKernelGGL(copy_status_rows_kernel, dim3(1), dim3(128), 0, s, src_status, dst_status, c);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// Pivot thresholds of the factorisation that tolerates dependent columns: a fraction of the Gram matrix' diagonal
__global__ void rank_threshold_kernel(void* const* table, int nslots, int rp, float tol) {
  void* const* tab = table + (size_t)blockIdx.y * nslots;
  const float* C = (const float*)tab[SLOT_C];
  float* thr = (float*)tab[SLOT_THR];
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < rp) thr[j] = tol * C[(long long)j * rp + j];
}
hipError_t launch_rank_threshold(void* const* table, int nslots, int batch, int rp, float tol, hipStream_t s) {
  if (batch <= 0) return hipSuccess;
  hipLaunchKernelGGL(rank_threshold_kernel, dim3((rp + 255) / 256, batch), dim3(256), 0, s, table, nslots, rp, tol);
  return hipGetLastError();
}

// Which matrices the fallback passes of the orthonormalisation have to redo (one thread per matrix)
__global__ void fallback_decide_kernel(void* const* table, int nslots, int batch) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= batch) return;
  void* const* tab = table + (size_t)i * nslots;
  int* status = (int*)tab[SLOT_STATUS];
  int* gate = (int*)tab[SLOT_GATE];
  if (*status == ST_BREAKDOWN) {
    *status = ST_OK;
    *gate = 0;
    *(int*)tab[SLOT_FAST] = 0;
  } else {
    *gate = 1;
  }
}
hipError_t launch_fallback_decide(void* const* table, int nslots, int batch, hipStream_t s) {
  if (batch <= 0) return hipSuccess;
  hipLaunchKernelGGL(fallback_decide_kernel, dim3((batch + 63) / 64), dim3(64), 0, s, table, nslots, batch);
  return hipGetLastError();
}

// ---------------------------------------------------------------- fills
__global__ void fill_kernel(void* const* table, int nslots, int slot, long long count, float value) {
  float* p = (float*)table[(size_t)blockIdx.y * nslots + slot];
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (long long)gridDim.x * blockDim.x)
    p[i] = value;
}
hipError_t launch_fill(void* const* table, int nslots, int batch, int slot, long long count, float value, hipStream_t s) {
  if (count <= 0 || batch <= 0) return hipSuccess;
  long long blocks = (count + 1023) / 1024;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(fill_kernel, dim3((unsigned)blocks, batch), dim3(256), 0, s, table, nslots, slot, count, value);
  return hipGetLastError();
}
// out <- in (count floats, a multiple of 4) unless the matrix' status word says that the step has failed
__global__ void copy_gated_kernel(void* const* table, int nslots, int slot_in, int slot_out, long long count, int status_slot) {
  void* const* tab = table + (size_t)blockIdx.y * nslots;
  if (status_slot >= 0 && *(const int*)tab[status_slot] != 0) return;
  const f32x4_t* in = (const f32x4_t*)tab[slot_in];
  f32x4_t* out = (f32x4_t*)tab[slot_out];
  const long long n4 = count >> 2;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (long long)gridDim.x * blockDim.x) out[i] = in[i];
  if (blockIdx.x == 0 && threadIdx.x < (count & 3)) ((float*)out)[n4 * 4 + threadIdx.x] = ((const float*)in)[n4 * 4 + threadIdx.x];
}
hipError_t launch_copy_gated(void* const* table, int nslots, int batch, int slot_in, int slot_out, long long count, int status_slot,
                             hipStream_t s) {
  if (count <= 0 || batch <= 0) return hipSuccess;
  long long blocks = (count / 4 + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(copy_gated_kernel, dim3((unsigned)blocks, batch), dim3(256), 0, s, table, nslots, slot_in, slot_out, count,
                     status_slot);
  return hipGetLastError();
}
__global__ void fill_i32_kernel(void* const* table, int nslots, int slot, long long count, int value) {
  int* p = (int*)table[(size_t)blockIdx.y * nslots + slot];
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (long long)gridDim.x * blockDim.x)
    p[i] = value;
}
hipError_t launch_fill_i32(void* const* table, int nslots, int batch, int slot, long long count, int value, hipStream_t s) {
  if (count <= 0 || batch <= 0) return hipSuccess;
  long long blocks = (count + 1023) / 1024;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)blocks, batch), dim3(256), 0, s, table, nslots, slot, count, value);
  return hipGetLastError();
}

// Gram matrix padding: rows/columns r..rp-1 of the rp x rp matrix become those of the identity, so
// that the Cholesky factor of the padded matrix is diag(L, I).
__global__ void pad_identity_kernel(void* const* table, int nslots, int slot, int r, int rp, int skip_slot) {
  if (skip_slot >= 0 && *(const int*)table[(size_t)blockIdx.y * nslots + skip_slot] != 0) return;
  float* p = (float*)table[(size_t)blockIdx.y * nslots + slot];
  const long long total = (long long)rp * rp;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    const int row = (int)(i / rp), col = (int)(i % rp);
    if (row >= r || col >= r) p[i] = (row == col) ? 1.f : 0.f;
  }
}
hipError_t launch_pad_identity(void* const* table, int nslots, int batch, int slot, int r, int rp, hipStream_t s, int skip_slot) {
  if (rp == r || batch <= 0) return hipSuccess;
  long long blocks = ((long long)rp * rp + 1023) / 1024;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(pad_identity_kernel, dim3((unsigned)blocks, batch), dim3(256), 0, s, table, nslots, slot, r, rp, skip_slot);
  return hipGetLastError();
}

__global__ void __launch_bounds__(256) shift_diagonal_kernel(void* const* table, int nslots, int r, int rp, float shift_rel, int skip_slot) {
  if (skip_slot >= 0 && *(const int*)table[(size_t)blockIdx.x * nslots + skip_slot] != 0) return;   // uniform, before any barrier
  float* C = (float*)table[(size_t)blockIdx.x * nslots + SLOT_C];
  __shared__ float red[256];
  float acc = 0.f;
  for (int j = threadIdx.x; j < r; j += 256) acc += C[(long long)j * rp + j];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int sft = 128; sft > 0; sft >>= 1) {
    if ((int)threadIdx.x < sft) red[threadIdx.x] += red[threadIdx.x + sft];
    __syncthreads();
  }
  const float shift = shift_rel * red[0];
  for (int j = threadIdx.x; j < r; j += 256) C[(long long)j * rp + j] += shift;
}
hipError_t launch_shift_diagonal(void* const* table, int nslots, int batch, int r, int rp, float shift_rel, hipStream_t s, int skip_slot) {
  hipLaunchKernelGGL(shift_diagonal_kernel, dim3(batch), dim3(256), 0, s, table, nslots, r, rp, shift_rel, skip_slot);
  return hipGetLastError();
}

// ---------------------------------------------------------------- split-K reduction (fixed order => deterministic)
// Sum of nsplit partial results `stride` floats apart, added in the order of the splits; eight loads are in flight
// at a time (a split beyond the last contributes +0, which changes no sum).
template <class T>
__device__ __forceinline__ T sum_planes(const float* p, long long stride, int nsplit) {
  T acc = T{};
  for (int sp = 0; sp < nsplit; sp += 8) {
    T v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = sp + u < nsplit ? gload<T>(p + (long long)(sp + u) * stride) : T{};
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u];
  }
  return acc;
}
// Lower triangle only (that is what is produced and consumed), in pieces of four columns: consecutive threads take
// consecutive pieces of a row, pieces above the diagonal are skipped.
__global__ void __launch_bounds__(256) reduce_partials_kernel(void* const* table, int nslots, int slot_part, int slot_out, int r,
                                                              long long ld, int nsplit, long long split_stride, int skip_slot) {
  if (skip_slot >= 0 && *(const int*)table[(size_t)blockIdx.y * nslots + skip_slot] != 0) return;
  const float* part = (const float*)table[(size_t)blockIdx.y * nslots + slot_part];
  float* out = (float*)table[(size_t)blockIdx.y * nslots + slot_out];
  const int ppr = (r + 3) / 4;   // pieces per row
  const long long total = (long long)r * ppr;
  for (long long w = (long long)blockIdx.x * 256 + threadIdx.x; w < total; w += (long long)gridDim.x * 256) {
    const int i = (int)(w / ppr), j0 = 4 * (int)(w % ppr);
    if (j0 > i) continue;
    const long long idx = (long long)i * ld + j0;
    if (j0 + 3 <= i) {
      gstore<f32x4_t>(out + idx, sum_planes<f32x4_t>(part + idx, split_stride, nsplit));
    } else {
      for (int j = j0; j <= i; ++j) out[idx + (j - j0)] = sum_planes<float>(part + idx + (j - j0), split_stride, nsplit);
    }
  }
}
hipError_t launch_reduce_partials(void* const* table, int nslots, int batch, int slot_part, int slot_out, int r, long long ld,
                                  int nsplit, long long split_stride, hipStream_t s, int skip_slot) {
  if (ld % 4 || split_stride % 4) return hipErrorInvalidValue;
  long long blocks = ((long long)r * ((r + 3) / 4) + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)blocks, batch), dim3(256), 0, s, table, nslots, slot_part, slot_out, r,
                     ld, nsplit, split_stride, skip_slot);
  return hipGetLastError();
}

__global__ void sum_partials_kernel(void* const* table, int nslots, int slot_part, int slot_out, long long count, int nsplit) {
  const f32x4_t* part = (const f32x4_t*)table[(size_t)blockIdx.y * nslots + slot_part];
  f32x4_t* out = (f32x4_t*)table[(size_t)blockIdx.y * nslots + slot_out];
  const long long n4 = count / 4;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (long long)gridDim.x * blockDim.x) {
    f32x4_t acc = part[i];
    for (int sp = 1; sp < nsplit; ++sp) acc += part[sp * n4 + i];
    out[i] = acc;
  }
}
hipError_t launch_sum_partials(void* const* table, int nslots, int batch, int slot_part, int slot_out, long long count,
                               int nsplit, hipStream_t s) {
  if (count % 4) return hipErrorInvalidValue;
  long long blocks = (count / 4 + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)blocks, batch), dim3(256), 0, s, table, nslots, slot_part, slot_out, count,
                     nsplit);
  return hipGetLastError();
}

// ---------------------------------------------------------------- ColNorm (update rule: V_new <- ColNorm(W))
// Stage 1: partial[chunk][col] = sum over the chunk's COLNORM_ROWS rows of in[row][col]^2.
__global__ void __launch_bounds__(256) colnorm_partial_kernel(void* const* table, int nslots, int slot_in, long long rows, int r) {
  const float* in = (const float*)table[(size_t)blockIdx.z * nslots + slot_in];
  float* part = (float*)table[(size_t)blockIdx.z * nslots + SLOT_SPART];
  __shared__ float red[4][64];
  const int cx = threadIdx.x & 63, ry = threadIdx.x >> 6;
  const int col = blockIdx.x * 64 + cx;
  const long long row_begin = (long long)blockIdx.y * COLNORM_ROWS;
  long long row_end = row_begin + COLNORM_ROWS;
  if (row_end > rows) row_end = rows;
  float acc = 0.f;
  if (col < r)
    for (long long row = row_begin + ry; row < row_end; row += 4) {
      const float v = in[row * r + col];
      acc += v * v;
    }
  red[ry][cx] = acc;
  __syncthreads();
  if (ry == 0 && col < r) part[(long long)blockIdx.y * r + col] = (red[0][cx] + red[1][cx]) + (red[2][cx] + red[3][cx]);
}
// Stage 2: s = sqrt(sum of partials), d = 1/(s + eps).  A block takes 64 columns; four threads share a column's
// chunks (chunk c goes to thread c mod 4) and their four sums are added in a fixed order.
__global__ void __launch_bounds__(256) colnorm_final_kernel(void* const* table, int nslots, int nchunks, int r) {
  const float* part = (const float*)table[(size_t)blockIdx.y * nslots + SLOT_SPART];
  float* sn = (float*)table[(size_t)blockIdx.y * nslots + SLOT_S];
  float* d = (float*)table[(size_t)blockIdx.y * nslots + SLOT_D];
  __shared__ float red[4][64];
  const int cx = threadIdx.x & 63, ry = threadIdx.x >> 6;
  const int col = blockIdx.x * 64 + cx;
  float acc = 0.f;
  if (col < r) {
    // eight loads in flight per thread (a single running sum would make the pass a chain of load latencies); the
    // order of the additions is fixed
    float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    int c = ry;
    for (; c + 28 < nchunks; c += 32) {
#pragma unroll
      for (int u = 0; u < 8; ++u) a[u] += part[(long long)(c + 4 * u) * r + col];
    }
    for (int u = 0; c < nchunks; c += 4, ++u) a[u] += part[(long long)c * r + col];
    acc = ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
  }
  red[ry][cx] = acc;
  __syncthreads();
  if (ry == 0 && col < r) {
    const float nrm = sqrtf((red[0][cx] + red[1][cx]) + (red[2][cx] + red[3][cx]));
    sn[col] = nrm;
    d[col] = 1.0f / (nrm + COLNORM_EPS);
  }
}
hipError_t launch_colnorm_final(void* const* table, int nslots, int batch, int nchunks, int r, hipStream_t s) {
  hipLaunchKernelGGL(colnorm_final_kernel, dim3((r + 63) / 64, batch), dim3(256), 0, s, table, nslots, nchunks, r);
  return hipGetLastError();
}
hipError_t launch_colnorm(void* const* table, int nslots, int batch, int slot_in, long long rows, int r, hipStream_t s) {
  const int nchunks = (int)((rows + COLNORM_ROWS - 1) / COLNORM_ROWS);
  hipLaunchKernelGGL(colnorm_partial_kernel, dim3((r + 63) / 64, nchunks, batch), dim3(256), 0, s, table, nslots, slot_in, rows, r);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(colnorm_final_kernel, dim3((r + 63) / 64, batch), dim3(256), 0, s, table, nslots, nchunks, r);
  return hipGetLastError();
}

// out[row][col] = in[row][col] * d[col]   (in may alias out).  Optionally also stores bf16 copies of the
// result (slot_out16) and of the input (slot_in16): the operands of the fused update kernel.
__global__ void __launch_bounds__(256) scale_cols_kernel(void* const* table, int nslots, int slot_in, int slot_out, long long rows,
                                                         int r, int status_slot, int slot_out16, int slot_in16, int null_slot) {
  void* const* tab = table + (size_t)blockIdx.z * nslots;
  if (status_slot >= 0 && *(const int*)tab[status_slot] != 0) return;
  const float* in = (const float*)tab[slot_in];
  float* out = (float*)tab[slot_out];
  uint16_t* out16 = slot_out16 >= 0 ? (uint16_t*)tab[slot_out16] : nullptr;
  uint16_t* in16 = slot_in16 >= 0 ? (uint16_t*)tab[slot_in16] : nullptr;
  const float* d = (const float*)tab[SLOT_D];
  const int* nullmask = null_slot >= 0 ? (const int*)tab[null_slot] : nullptr;
  // a block covers 64 rows x 256 columns; a thread owns 4 consecutive columns (or fewer at a ragged edge)
  const int col = blockIdx.x * 256 + (threadIdx.x & 63) * 4;
  if (col >= r) return;
  const long long row_end = min(rows, ((long long)blockIdx.y + 1) * 64);
  if ((r & 3) == 0) {
    const f32x4_t dv = *(const f32x4_t*)(d + col);
    bool keep_old[4] = {false, false, false, false};
    bool any_old = false;
    if (nullmask) {
#pragma unroll
      for (int e = 0; e < 4; ++e) { keep_old[e] = nullmask[col + e] != 0; any_old = any_old || keep_old[e]; }
    }
    for (long long row = (long long)blockIdx.y * 64 + (threadIdx.x >> 6); row < row_end; row += 4) {
      const long long idx = row * r + col;
      const f32x4_t v = *(const f32x4_t*)(in + idx);
      const f32x4_t q = v * dv;
      if (any_old) {
        f32x4_t o = *(const f32x4_t*)(out + idx);
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = keep_old[e] ? o[e] : q[e];
        *(f32x4_t*)(out + idx) = o;
      } else {
        *(f32x4_t*)(out + idx) = q;
      }
      if (out16) { u32x2_t w = {pack_bf16x2(q[0], q[1]), pack_bf16x2(q[2], q[3])}; *(u32x2_t*)(out16 + idx) = w; }
      if (in16) { u32x2_t w = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])}; *(u32x2_t*)(in16 + idx) = w; }
    }
  } else {
    for (long long row = (long long)blockIdx.y * 64 + (threadIdx.x >> 6); row < row_end; row += 4)
      for (int c = col; c < min(col + 4, r); ++c) {
        const long long idx = row * r + c;
        const float v = in[idx];
        const float q = v * d[c];
        if (!(nullmask && nullmask[c] != 0)) out[idx] = q;
        if (out16) out16[idx] = (uint16_t)(pack_bf16x2(q, 0.f) & 0xffffu);
        if (in16) in16[idx] = (uint16_t)(pack_bf16x2(v, 0.f) & 0xffffu);
      }
  }
}
hipError_t launch_scale_cols(void* const* table, int nslots, int batch, int slot_in, int slot_out, long long rows, int r,
                             int status_slot, int slot_out16, int slot_in16, hipStream_t s, int null_slot) {
  hipLaunchKernelGGL(scale_cols_kernel, dim3((r + 255) / 256, (unsigned)((rows + 63) / 64), batch), dim3(256), 0, s, table, nslots,
                     slot_in, slot_out, rows, r, status_slot, slot_out16, slot_in16, null_slot);
  return hipGetLastError();
}

// fp32 [rows][cols] -> bf16 [rows][cols] and / or bf16 [cols][rows], 64x64 tiles transposed through LDS.
// skip_slot >= 0 and the int32 there non-zero: nothing to do.
__global__ void __launch_bounds__(256) convert_bf16_kernel(void* const* table, int nslots, int slot_in, int slot_out16,
                                                           int slot_outT16, long long rows, long long cols, int skip_slot) {
  void* const* tab = table + (size_t)blockIdx.z * nslots;
  if (skip_slot >= 0 && *(const int*)tab[skip_slot] != 0) return;
  const float* in = (const float*)tab[slot_in];
  uint16_t* out16 = slot_out16 >= 0 ? (uint16_t*)tab[slot_out16] : nullptr;
  uint16_t* outT = slot_outT16 >= 0 ? (uint16_t*)tab[slot_outT16] : nullptr;
  __shared__ float tile[64][65];
  const long long row0 = (long long)blockIdx.y * 64, col0 = (long long)blockIdx.x * 64;
  const int t = threadIdx.x;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int rr = p * 16 + (t >> 4), c4 = (t & 15) * 4;
    const f32x4_t v = *(const f32x4_t*)(in + (row0 + rr) * cols + col0 + c4);
    tile[rr][c4 + 0] = v[0]; tile[rr][c4 + 1] = v[1]; tile[rr][c4 + 2] = v[2]; tile[rr][c4 + 3] = v[3];
    if (out16) {
      u32x2_t w = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
      *(u32x2_t*)(out16 + (row0 + rr) * cols + col0 + c4) = w;
    }
  }
  if (!outT) return;
  __syncthreads();
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int cc = p * 16 + (t >> 4), r4 = (t & 15) * 4;
    u32x2_t w = {pack_bf16x2(tile[r4 + 0][cc], tile[r4 + 1][cc]), pack_bf16x2(tile[r4 + 2][cc], tile[r4 + 3][cc])};
    *(u32x2_t*)(outT + (col0 + cc) * rows + row0 + r4) = w;
  }
}
hipError_t launch_convert_bf16(void* const* table, int nslots, int batch, int slot_in, int slot_out16, int slot_outT16,
                               long long rows, long long cols, hipStream_t s, int skip_slot) {
  if (rows % 64 || cols % 64) return hipErrorInvalidValue;
  hipLaunchKernelGGL(convert_bf16_kernel, dim3((unsigned)(cols / 64), (unsigned)(rows / 64), batch), dim3(256), 0, s, table, nslots,
                     slot_in, slot_out16, slot_outT16, rows, cols, skip_slot);
  return hipGetLastError();
}

// bf16(M + G), row-major: the accumulated buffer B = M + G of the step (Algorithm 1) rounded once to the operand
// precision of the bf16 products; B Q reads it with its contraction index contiguous, B^T P with that index as the
// slow one.  A plain streaming pass, eight elements per thread and step (32 + 16 bytes in, 16 bytes out), nothing
// through LDS.
template <bool GBF16>
__global__ void __launch_bounds__(256) sum_bf16_stream_kernel(void* const* table, int nslots, int slot_m, int slot_g, int slot_out16,
                                                              long long count8) {
  void* const* tab = table + (size_t)blockIdx.y * nslots;
  const f32x4_t* M = (const f32x4_t*)tab[slot_m];
  const void* G = tab[slot_g];
  u32x4_t* out = (u32x4_t*)tab[slot_out16];
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < count8; i += stride) {
    f32x4_t a = M[2 * i], b = M[2 * i + 1];
    if constexpr (GBF16) {
      const u32x4_t w = ((const u32x4_t*)G)[i];
      a += f32x4_t{bf16_lo(w[0]), bf16_hi(w[0]), bf16_lo(w[1]), bf16_hi(w[1])};
      b += f32x4_t{bf16_lo(w[2]), bf16_hi(w[2]), bf16_lo(w[3]), bf16_hi(w[3])};
    } else {
      a += ((const f32x4_t*)G)[2 * i];
      b += ((const f32x4_t*)G)[2 * i + 1];
    }
    out[i] = u32x4_t{pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(b[0], b[1]), pack_bf16x2(b[2], b[3])};
  }
}
// The same for the columns [8 c8_first, 8 (c8_first + c8_count)) of the rows [row_first, row_first + rows) only
// (cols8 = columns / 8): one part of the copy, so that the product over the part before it can run meanwhile.
template <bool GBF16>
__global__ void __launch_bounds__(256) sum_bf16_cols_kernel(void* const* table, int nslots, int slot_m, int slot_g, int slot_out16,
                                                            long long row_first, long long rows, long long cols8, long long c8_first,
                                                            long long c8_count) {
  void* const* tab = table + (size_t)blockIdx.y * nslots;
  const f32x4_t* M = (const f32x4_t*)tab[slot_m];
  const void* G = tab[slot_g];
  u32x4_t* out = (u32x4_t*)tab[slot_out16];
  const long long stride = (long long)gridDim.x * blockDim.x, total = rows * c8_count;
  for (long long w = (long long)blockIdx.x * blockDim.x + threadIdx.x; w < total; w += stride) {
    const long long row = w / c8_count, i = (row_first + row) * cols8 + c8_first + (w - row * c8_count);
    f32x4_t a = gload_nt<f32x4_t>(M + 2 * i), b = gload_nt<f32x4_t>(M + 2 * i + 1);
    if constexpr (GBF16) {
      const u32x4_t g4 = gload_nt<u32x4_t>((const u32x4_t*)G + i);
      a += f32x4_t{bf16_lo(g4[0]), bf16_hi(g4[0]), bf16_lo(g4[1]), bf16_hi(g4[1])};
      b += f32x4_t{bf16_lo(g4[2]), bf16_hi(g4[2]), bf16_lo(g4[3]), bf16_hi(g4[3])};
    } else {
      a += ((const f32x4_t*)G)[2 * i];
      b += ((const f32x4_t*)G)[2 * i + 1];
    }
    gstore_nt<u32x4_t>(out + i, u32x4_t{pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(b[0], b[1]), pack_bf16x2(b[2], b[3])});
  }
}
hipError_t launch_sum_bf16_cols(void* const* table, int nslots, int batch, int slot_m, int slot_g, bool gbf16, int slot_out16,
                                long long rows, long long cols, long long row_first, long long row_count, long long col_first,
                                long long col_count, hipStream_t s) {
  if (cols % 8 || col_first % 8 || col_count % 8 || col_first < 0 || col_count < 1 || col_first + col_count > cols || batch > 65535 ||
      batch < 1 || row_first < 0 || row_count < 1 || row_first + row_count > rows)
    return hipErrorInvalidValue;
  const long long total = row_count * (col_count / 8);
  long long blocks = (total + 255) / 256;
  // Many short-lived workgroups (one or two steps per thread) and non-temporal accesses: this pass runs beside a product,
  // and that is how it disturbs it least (C4 r = 1024, the K1 stage: 2.59 ms with 4097 workgroups per launch, 2.43 ms with
  // 65537; plain accesses instead of hinted ones: + 0.15 ms)
  const long long cap = 256LL * 256 / (batch < 16 ? batch : 16) + 1;
  if (blocks > cap) blocks = cap;
  const dim3 grid((unsigned)blocks, batch);
  if (gbf16) hipLaunchKernelGGL(sum_bf16_cols_kernel<true>, grid, dim3(256), 0, s, table, nslots, slot_m, slot_g, slot_out16, row_first, row_count, cols / 8, col_first / 8, col_count / 8);
  else hipLaunchKernelGGL(sum_bf16_cols_kernel<false>, grid, dim3(256), 0, s, table, nslots, slot_m, slot_g, slot_out16, row_first, row_count, cols / 8, col_first / 8, col_count / 8);
  return hipGetLastError();
}
hipError_t launch_sum_bf16(void* const* table, int nslots, int batch, int slot_m, int slot_g, bool gbf16, int slot_out16,
                           long long rows, long long cols, hipStream_t s) {
  if (rows * cols % 8 || batch > 65535 || batch < 1) return hipErrorInvalidValue;
  const long long count8 = rows * cols / 8;
  long long blocks = (count8 + 255) / 256;
  const long long cap = 256LL * 64 / (batch < 64 ? batch : 64) + 1;   // about 64 workgroups per compute unit over the whole launch
  if (blocks > cap) blocks = cap;
  const dim3 grid((unsigned)blocks, batch);
  if (gbf16) hipLaunchKernelGGL(sum_bf16_stream_kernel<true>, grid, dim3(256), 0, s, table, nslots, slot_m, slot_g, slot_out16, count8);
  else hipLaunchKernelGGL(sum_bf16_stream_kernel<false>, grid, dim3(256), 0, s, table, nslots, slot_m, slot_g, slot_out16, count8);
  return hipGetLastError();
}

// x = hi + lo with hi = bf16(x), lo = bf16(x - hi): the three products hi*hi + hi*lo + lo*hi then carry about
// 16 mantissa bits on the bf16 matrix pipe.
__global__ void __launch_bounds__(256) split_bf16_kernel(void* const* table, int nslots, int slot_in, long long ld_in,
                                                         long long rows, long long cols, int slot_hi, int slot_lo,
                                                         int slot_hiT, int slot_loT, int skip_slot) {
  void* const* tab = table + (size_t)blockIdx.z * nslots;
  if (skip_slot >= 0 && *(const int*)tab[skip_slot] != 0) return;
  const float* in = (const float*)tab[slot_in];
  uint16_t* hi = slot_hi >= 0 ? (uint16_t*)tab[slot_hi] : nullptr;
  uint16_t* lo = slot_lo >= 0 ? (uint16_t*)tab[slot_lo] : nullptr;
  uint16_t* hiT = slot_hiT >= 0 ? (uint16_t*)tab[slot_hiT] : nullptr;
  uint16_t* loT = slot_loT >= 0 ? (uint16_t*)tab[slot_loT] : nullptr;
  __shared__ uint32_t tile[64][65];   // (lo << 16) | hi per element
  const long long row0 = (long long)blockIdx.y * 64, col0 = (long long)blockIdx.x * 64;
  const int t = threadIdx.x;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int rr = p * 16 + (t >> 4), c4 = (t & 15) * 4;
    const f32x4_t v = *(const f32x4_t*)(in + (row0 + rr) * ld_in + col0 + c4);
    uint32_t h[4], l[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      h[e] = pack_bf16x2(v[e], 0.f) & 0xffffu;
      l[e] = pack_bf16x2(v[e] - bf16_to_f32((uint16_t)h[e]), 0.f) & 0xffffu;
      tile[rr][c4 + e] = (l[e] << 16) | h[e];
    }
    if (hi) { u32x2_t w = {h[0] | (h[1] << 16), h[2] | (h[3] << 16)}; *(u32x2_t*)(hi + (row0 + rr) * cols + col0 + c4) = w; }
    if (lo) { u32x2_t w = {l[0] | (l[1] << 16), l[2] | (l[3] << 16)}; *(u32x2_t*)(lo + (row0 + rr) * cols + col0 + c4) = w; }
  }
  if (!hiT && !loT) return;
  __syncthreads();
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int cc = p * 16 + (t >> 4), r4 = (t & 15) * 4;
    const uint32_t e0 = tile[r4 + 0][cc], e1 = tile[r4 + 1][cc], e2 = tile[r4 + 2][cc], e3 = tile[r4 + 3][cc];
    if (hiT) { u32x2_t w = {(e0 & 0xffffu) | (e1 << 16), (e2 & 0xffffu) | (e3 << 16)}; *(u32x2_t*)(hiT + (col0 + cc) * rows + row0 + r4) = w; }
    if (loT) { u32x2_t w = {(e0 >> 16) | (e1 & 0xffff0000u), (e2 >> 16) | (e3 & 0xffff0000u)}; *(u32x2_t*)(loT + (col0 + cc) * rows + row0 + r4) = w; }
  }
}
hipError_t launch_split_bf16(void* const* table, int nslots, int batch, int slot_in, long long ld_in, long long rows,
                             long long cols, int slot_hi, int slot_lo, int slot_hiT, int slot_loT, hipStream_t s, int skip_slot) {
  if (rows % 64 || cols % 64 || ld_in % 4) return hipErrorInvalidValue;
  hipLaunchKernelGGL(split_bf16_kernel, dim3((unsigned)(cols / 64), (unsigned)(rows / 64), batch), dim3(256), 0, s, table, nslots,
                     slot_in, ld_in, rows, cols, slot_hi, slot_lo, slot_hiT, slot_loT, skip_slot);
  return hipGetLastError();
}

// ---------------------------------------------------------------- first-order inverse Cholesky factor near the identity
// nsplit > 1: the Gram matrix arrives as split-K partial results (SLOT_CPART, split_stride apart); their sum, taken in the
// fixed order, is stored to SLOT_C on the way.
__global__ void __launch_bounds__(256) gram_defect_kernel(void* const* table, int nslots, int r, long long ld, int nsplit,
                                                          long long split_stride) {
  void* const* tab = table + (size_t)blockIdx.y * nslots;
  float* C = (float*)tab[SLOT_C];
  const float* cpart = (const float*)tab[SLOT_CPART];
  float* part = (float*)tab[SLOT_EPART];
  __shared__ float red[256];
  float acc = 0.f;
  // the lower triangle in pieces of four columns, consecutive threads on consecutive pieces of a row
  const int ppr = (r + 3) / 4;
  const long long total = (long long)r * ppr;
  for (long long w = (long long)blockIdx.x * 256 + threadIdx.x; w < total; w += (long long)gridDim.x * 256) {
    const int i = (int)(w / ppr), j0 = 4 * (int)(w % ppr);
    if (j0 > i) continue;
    const long long idx = (long long)i * ld + j0;
    if (j0 + 3 <= i) {
      f32x4_t c;
      if (nsplit > 1) {
        c = sum_planes<f32x4_t>(cpart + idx, split_stride, nsplit);
        gstore<f32x4_t>(C + idx, c);
      } else {
        c = gload<f32x4_t>(C + idx);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool diag = j0 + e == i;
        const float d = c[e] - (diag ? 1.f : 0.f);
        acc += (diag ? 1.f : 2.f) * d * d;
      }
    } else {
      for (int j = j0; j <= i; ++j) {
        float c;
        if (nsplit > 1) {
          c = sum_planes<float>(cpart + idx + (j - j0), split_stride, nsplit);
          C[idx + (j - j0)] = c;
        } else {
          c = C[idx + (j - j0)];
        }
        const float d = c - (i == j ? 1.f : 0.f);
        acc += (i == j ? 1.f : 2.f) * d * d;
      }
    }
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int sft = 128; sft > 0; sft >>= 1) {
    if ((int)threadIdx.x < sft) red[threadIdx.x] += red[threadIdx.x + sft];
    __syncthreads();
  }
  if (threadIdx.x == 0) part[blockIdx.x] = red[0];
}
__global__ void __launch_bounds__(256) first_order_inverse_kernel(void* const* table, int nslots, int r, int rp, float tau2,
                                                                  int decision_only) {
  void* const* tab = table + (size_t)blockIdx.y * nslots;
  const float* part = (const float*)tab[SLOT_EPART];
  // every block adds the partials in the same order, so all blocks take the same decision
  __shared__ float red[256];
  {
    float acc = 0.f;
    for (int k = threadIdx.x; k < GRAM_DEFECT_PARTS; k += 256) acc += part[k];
    red[threadIdx.x] = acc;
  }
  __syncthreads();
  for (int sft = 128; sft > 0; sft >>= 1) {
    if ((int)threadIdx.x < sft) red[threadIdx.x] += red[threadIdx.x + sft];
    __syncthreads();
  }
  const float total = red[0];
  const bool fast = total <= tau2;   // false for NaN
  if (blockIdx.x == 0 && threadIdx.x == 0) *(int*)tab[SLOT_FAST] = fast ? 1 : 0;
  if (!fast || decision_only) return;
  const float* C = (const float*)tab[SLOT_C];
  float* W = (float*)tab[SLOT_W];
  const long long n = (long long)rp * rp;
  for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < n; idx += (long long)gridDim.x * 256) {
    const int i = (int)(idx / rp), j = (int)(idx % rp);
    float v = 0.f, phi = 0.f;
    if (i < r && j < r) {
      if (i == j) phi = 0.5f * (C[idx] - 1.f);
      else if (j < i) phi = C[idx];
      v = (i == j ? 1.f : 0.f) - phi;
    } else if (i == j) {
      v = 1.f;
    }
    W[idx] = v;
  }
}
hipError_t launch_first_order_inverse(void* const* table, int nslots, int batch, int r, int rp, float tau, bool decision_only,
                                      int nsplit, long long split_stride, hipStream_t s) {
  if (rp % 4 || split_stride % 4) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gram_defect_kernel, dim3(GRAM_DEFECT_PARTS, batch), dim3(256), 0, s, table, nslots, r, (long long)rp, nsplit,
                     split_stride);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  long long blocks = ((long long)rp * rp + 2047) / 2048;
  if (blocks > 1024) blocks = 1024;
  if (decision_only) blocks = 1;
  hipLaunchKernelGGL(first_order_inverse_kernel, dim3((unsigned)blocks, batch), dim3(256), 0, s, table, nslots, r, rp, tau * tau,
                     decision_only ? 1 : 0);
  return hipGetLastError();
}

// ---------------------------------------------------------------- Gaussian fill (Philox-4x32-10 + Box-Muller)
__device__ __forceinline__ void philox_round(uint32_t (&c)[4], uint32_t k0, uint32_t k1) {
  const uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
  const uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
  const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0;
  const uint32_t n1 = (uint32_t)p1;
  const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
  const uint32_t n3 = (uint32_t)p0;
  c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
}
// Element e comes from block e/4 (counter = (block lo, block hi, stream, 0), key = seed): words (0,1)
// and (2,3) feed two Box-Muller transforms, u1 = (w+1)/2^32, u2 = w'/2^32.
__global__ void gaussian_fill_kernel(void* const* table, int nslots, int slot, long long count, uint64_t seed, int first_stream) {
  float* out = (float*)table[(size_t)blockIdx.y * nslots + slot];
  const long long nblk = (count + 3) / 4;
  for (long long blk = (long long)blockIdx.x * blockDim.x + threadIdx.x; blk < nblk; blk += (long long)gridDim.x * blockDim.x) {
    uint32_t c[4] = {(uint32_t)blk, (uint32_t)((uint64_t)blk >> 32), (uint32_t)(first_stream + blockIdx.y), 0u};
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
    for (int rd = 0; rd < 10; ++rd) {
      philox_round(c, k0, k1);
      k0 += 0x9E3779B9u;
      k1 += 0xBB67AE85u;
    }
    float v[4];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const double u1 = ((double)c[2 * h] + 1.0) * (1.0 / 4294967296.0);
      const double u2 = (double)c[2 * h + 1] * (1.0 / 4294967296.0);
      const double rad = sqrt(-2.0 * log(u1));
      double sn, cs;
      sincos(6.283185307179586476925286766559 * u2, &sn, &cs);
      v[2 * h] = (float)(rad * cs);
      v[2 * h + 1] = (float)(rad * sn);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (blk * 4 + e < count) out[blk * 4 + e] = v[e];
  }
}
hipError_t launch_gaussian_fill(void* const* table, int nslots, int batch, int slot, long long count, uint64_t seed,
                                int first_stream, hipStream_t s) {
  if (count <= 0 || batch <= 0) return hipSuccess;
  long long blocks = ((count + 3) / 4 + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(gaussian_fill_kernel, dim3((unsigned)blocks, batch), dim3(256), 0, s, table, nslots, slot, count, seed,
                     first_stream);
  return hipGetLastError();
}

}  // namespace dion
