// Two micro-kernels that measure what this GPU delivers for the two resources the step's rooflines are written
// against, so that a benchmark run can quote achieved rates against measured ceilings as well as published peaks:
//   an issue-only loop of v_mfma_f32_32x32x16_bf16 (no memory traffic), and
//   a streaming pass with the traffic pattern of the fused update's epilogue: read fp32, bf16, fp32; write fp32, fp32.
#include "internal.hpp"
namespace dion {

__global__ void __launch_bounds__(512, 1) probe_mfma_kernel(float* sink, int iters) {
  bf16x8_t a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)(threadIdx.x & 3); b[e] = (__bf16)1.0f; }
  f32x16_t acc[8];
#pragma unroll
  for (int q = 0; q < 8; ++q)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[q][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[q], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int q = 0; q < 8; ++q) s += acc[q][0];
  if (s == -1.f) sink[0] = s;   // never true: keeps the loop alive
}

// a[i] = a[i] + g[i] - 0.5 x[i];  x[i] = x[i] - 0.25 a_old[i]   (18 bytes per element, 16-byte accesses, with or
// without the non-temporal hint)
template <bool NT>
__global__ void __launch_bounds__(256) probe_stream_kernel(float* a, const uint16_t* g, float* x, long long n4) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    const f32x4_t av = NT ? gload_nt<f32x4_t>(a + 4 * i) : gload<f32x4_t>(a + 4 * i);
    const f32x4_t xv = NT ? gload_nt<f32x4_t>(x + 4 * i) : gload<f32x4_t>(x + 4 * i);
    const u32x2_t w = NT ? gload_nt<u32x2_t>(g + 4 * i) : gload<u32x2_t>(g + 4 * i);
    const f32x4_t gv = {bf16_lo(w[0]), bf16_hi(w[0]), bf16_lo(w[1]), bf16_hi(w[1])};
    const f32x4_t na = av + gv - 0.5f * xv, nx = xv - 0.25f * av;
    if (NT) {
      gstore_nt<f32x4_t>(a + 4 * i, na);
      gstore_nt<f32x4_t>(x + 4 * i, nx);
    } else {
      gstore<f32x4_t>(a + 4 * i, na);
      gstore<f32x4_t>(x + 4 * i, nx);
    }
  }
}

// Times both on `s` with events (this call synchronises).  scratch: at least 10 * elems bytes, 256-byte aligned;
// its contents are used as they are (the rates do not depend on the values).
hipError_t run_ceiling_probes(void* scratch, long long elems, double* mfma_tflops, double* stream_gbps, hipStream_t s) {
  hipEvent_t e0, e1;
  hipError_t e = hipEventCreate(&e0);
  if (e != hipSuccess) return e;
  e = hipEventCreate(&e1);
  if (e != hipSuccess) { (void)hipEventDestroy(e0); return e; }
  auto fail = [&](hipError_t err) { (void)hipEventDestroy(e0); (void)hipEventDestroy(e1); return err; };
  float ms = 0.f;
  // MFMA: 1024 workgroups of 8 waves, 8 independent accumulators per wave
  const int iters = 2000, groups = 1024;
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(groups), dim3(512), 0, s, (float*)scratch, 10);   // warm-up
  if ((e = hipEventRecord(e0, s)) != hipSuccess) return fail(e);
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(groups), dim3(512), 0, s, (float*)scratch, iters);
  if ((e = hipEventRecord(e1, s)) != hipSuccess) return fail(e);
  if ((e = hipEventSynchronize(e1)) != hipSuccess) return fail(e);
  if ((e = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess) return fail(e);
  *mfma_tflops = (double)groups * 8 * 8 * iters * (2.0 * 32 * 32 * 16) / (ms * 1e-3) * 1e-12;
  // stream: a (fp32), x (fp32), g (bf16) carved from scratch
  // whole multiples of 2^20 elements, so that the three arrays start on the same alignment as the first (an odd size
  // that leaves the second array 16 bytes into a 256-byte line measured 10 % lower), and no more than 2^26, the
  // matrix size of the 8192 x 8192 workload: the rate is the best case for footprints of that size and more (0.67 GB
  // keeps a larger share of itself in the 256 MB last-level cache between passes than 1 GB does, which streams
  // about 10 % slower)
  long long n = elems / (1 << 20) * (1 << 20);
  if (n > (1ll << 26)) n = 1ll << 26;
  if (n <= 0) return hipErrorInvalidValue;
  float* a = (float*)scratch;
  float* x = a + n;
  uint16_t* g = (uint16_t*)(x + n);
  // the best of a few grid sizes and of both kinds of access counts: a ceiling must not be understated by an unlucky
  // launch shape
  *stream_gbps = 0.0;
  const int grids[5] = {1024, 2048, 4096, 8192, 16384};
  for (int gi = 0; gi < 10; ++gi) {
    const dim3 grid(grids[gi % 5]);
    auto launch = [&] {
      if (gi < 5) hipLaunchKernelGGL(probe_stream_kernel<false>, grid, dim3(256), 0, s, a, g, x, n / 4);
      else hipLaunchKernelGGL(probe_stream_kernel<true>, grid, dim3(256), 0, s, a, g, x, n / 4);
    };
    launch();   // warm-up
    if ((e = hipEventRecord(e0, s)) != hipSuccess) return fail(e);
    for (int rep = 0; rep < 4; ++rep) launch();
    if ((e = hipEventRecord(e1, s)) != hipSuccess) return fail(e);
    if ((e = hipEventSynchronize(e1)) != hipSuccess) return fail(e);
    if ((e = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess) return fail(e);
    const double rate = 4.0 * 18.0 * (double)n / (ms * 1e-3) * 1e-9;
    if (rate > *stream_gbps) *stream_gbps = rate;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return hipGetLastError();
}

}  // namespace dion
